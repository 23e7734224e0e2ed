// (dtype, op) instantiations: 64-bit integers.
#include "ks_launch.hpp"

namespace ks {
const PairEntry *pair_entry_i64(int dtype, int op) {
    if (dtype == KS_I64) {
        if (op == KS_SUM) return Pair<int64_t, SumOp<int64_t>>::entry();
        if (op == KS_MIN) return Pair<int64_t, MinOp<int64_t>>::entry();
        if (op == KS_MAX) return Pair<int64_t, MaxOp<int64_t>>::entry();
    }
    if (dtype == KS_U64) {
        if (op == KS_SUM) return Pair<uint64_t, SumOp<uint64_t>>::entry();
        if (op == KS_MIN) return Pair<uint64_t, MinOp<uint64_t>>::entry();
        if (op == KS_MAX) return Pair<uint64_t, MaxOp<uint64_t>>::entry();
    }
    return nullptr;
}
}  // namespace ks
