// (dtype, map, op) instantiations of the map-fused scan, scan(f, op, src) of the
// paper's Sec. IV-A.  Each one is compiled in the shapes its element class's defaults can select.
#include "ks_launch.hpp"

namespace ks {
const PairEntry *pair_entry_mapped(int dtype, int map, int op) {
    if (dtype == KS_F32) {
        if (map == KS_MAP_SQUARE && op == KS_SUM) return Pair<float, MappedOp<SumOp<float>, SquareMap>>::entry();
        if (map == KS_MAP_ABS && op == KS_SUM) return Pair<float, MappedOp<SumOp<float>, AbsMap>>::entry();
        if (map == KS_MAP_ABS && op == KS_MAX) return Pair<float, MappedOp<MaxOp<float>, AbsMap>>::entry();
    }
    if (dtype == KS_F64) {
        if (map == KS_MAP_SQUARE && op == KS_SUM) return Pair<double, MappedOp<SumOp<double>, SquareMap>>::entry();
    }
    if (dtype == KS_I32) {
        if (map == KS_MAP_NONZERO && op == KS_SUM) return Pair<int32_t, MappedOp<SumOp<int32_t>, NonzeroMap>>::entry();
        if (map == KS_MAP_ABS && op == KS_MAX) return Pair<int32_t, MappedOp<MaxOp<int32_t>, AbsMap>>::entry();
        if (map == KS_MAP_SQUARE && op == KS_SUM) return Pair<int32_t, MappedOp<SumOp<int32_t>, SquareMap>>::entry();
    }
    if (dtype == KS_U64) {
        if (map == KS_MAP_NONZERO && op == KS_SUM) return Pair<uint64_t, MappedOp<SumOp<uint64_t>, NonzeroMap>>::entry();
    }
    return nullptr;
}
}  // namespace ks
