// (dtype, op) instantiations: float and double.
#include "ks_launch.hpp"

namespace ks {
const PairEntry *pair_entry_float(int dtype, int op) {
    if (dtype == KS_F32) {
        if (op == KS_SUM) return Pair<float, SumOp<float>>::entry();
        if (op == KS_MIN) return Pair<float, MinOp<float>>::entry();
        if (op == KS_MAX) return Pair<float, MaxOp<float>>::entry();
    }
    if (dtype == KS_F64) {
        if (op == KS_SUM) return Pair<double, SumOp<double>>::entry();
        if (op == KS_MIN) return Pair<double, MinOp<double>>::entry();
        if (op == KS_MAX) return Pair<double, MaxOp<double>>::entry();
    }
    return nullptr;
}
}  // namespace ks
