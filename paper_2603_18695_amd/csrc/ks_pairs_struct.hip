// (dtype, op) instantiations: composite element types.
#include "ks_launch.hpp"

namespace ks {
const PairEntry *pair_entry_struct(int dtype, int op) {
    if (dtype == KS_AFFINE_F32 && op == KS_AFFINE_COMPOSE) return Pair<AffineF32, AffineComposeOp>::entry();
    if (dtype == KS_ARGMAX_I32_CNT64 && op == KS_ARGMAX_COUNT) return Pair<ArgmaxI32Cnt64, ArgmaxCountOp>::entry();
    if (dtype == KS_MAT2_U32 && op == KS_MAT2_MUL) return Pair<Mat2U32, Mat2MulOp>::entry();
    if (dtype == KS_QUAT_F32 && op == KS_QUAT_MUL) return Pair<QuatF32, QuatMulOp>::entry();
    if (dtype == KS_MAT2_U64 && op == KS_MAT2_MUL) return Pair<Mat2U64, Mat2WideMulOp>::entry();
    if (dtype == KS_RANGE_I32_CNT32 && op == KS_RANGE_COUNT) return Pair<RangeI32Cnt32, RangeCountOp>::entry();
    return nullptr;
}
}  // namespace ks
