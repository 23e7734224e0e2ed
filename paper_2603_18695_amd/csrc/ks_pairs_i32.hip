// (dtype, op) instantiations: 32-bit integers.
#include "ks_launch.hpp"

namespace ks {
const PairEntry *pair_entry_i32(int dtype, int op) {
    if (dtype == KS_I32) {
        if (op == KS_SUM) return Pair<int32_t, SumOp<int32_t>>::entry();
        if (op == KS_MIN) return Pair<int32_t, MinOp<int32_t>>::entry();
        if (op == KS_MAX) return Pair<int32_t, MaxOp<int32_t>>::entry();
    }
    if (dtype == KS_U32) {
        if (op == KS_SUM) return Pair<uint32_t, SumOp<uint32_t>>::entry();
        if (op == KS_MIN) return Pair<uint32_t, MinOp<uint32_t>>::entry();
        if (op == KS_MAX) return Pair<uint32_t, MaxOp<uint32_t>>::entry();
    }
    return nullptr;
}
}  // namespace ks
