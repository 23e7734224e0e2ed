// Reductions over bytes: the 8-bit element types of the paper's mapreduce benchmark
// (Sec. VII-B; Tables I and III: UnitFloat8 promoted to Float32, and raw UInt8).
#include "ks_launch.hpp"

namespace ks {
const PairEntry *pair_entry_bytes(int dtype, int map, int op) {
    if (dtype != KS_U8 || op != KS_SUM) return nullptr;
    if (map == KS_MAP_UNIT_FLOAT8) return ReducePair<uint8_t, MappedOp<SumOp<float>, UnitFloat8Map>>::entry();
    if (map == KS_MAP_WIDEN64) return ReducePair<uint8_t, MappedOp<ByteWideSumOp, Widen64Map>>::entry();
    if (map == KS_MAP_IDENTITY) return ReducePair<uint8_t, ByteSumOp>::entry();
    return nullptr;
}
}  // namespace ks
