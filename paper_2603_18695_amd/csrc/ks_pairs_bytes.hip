// Reductions over elements narrower than the scan kernels' 4 bytes: the 8-bit types of the paper's
// mapreduce benchmark (Sec. VII-B; Tables I and III: UnitFloat8 promoted to Float32, and raw UInt8),
// and 16-bit floats promoted to float32 the same way.
#include "ks_launch.hpp"

namespace ks {
template <class T>
static const PairEntry *half_entry(int op) {
    if (op == KS_SUM) return ReducePair<T, MappedOp<SumOp<float>, WidenF32Map>>::entry();
    if (op == KS_MIN) return ReducePair<T, MappedOp<MinOp<float>, WidenF32Map>>::entry();
    if (op == KS_MAX) return ReducePair<T, MappedOp<MaxOp<float>, WidenF32Map>>::entry();
    return nullptr;
}

// Scans of 16-bit floats: every element promoted to float32 as it is loaded, accumulated in float32
// (sums: double above one wave's run), every output rounded to the 16-bit type, ties to even.
template <class T>
static const PairEntry *half_scan_entry(int op) {
    if (op == KS_SUM) return Pair<T, MappedOp<SumOp<float>, WidenF32Map>>::entry();
    if (op == KS_MIN) return Pair<T, MappedOp<MinOp<float>, WidenF32Map>>::entry();
    if (op == KS_MAX) return Pair<T, MappedOp<MaxOp<float>, WidenF32Map>>::entry();
    return nullptr;
}
const PairEntry *pair_entry_half(int dtype, int op) {
    if (dtype == KS_BF16) return half_scan_entry<BF16Bits>(op);
    if (dtype == KS_F16) return half_scan_entry<F16Bits>(op);
    return nullptr;
}

const PairEntry *pair_entry_bytes(int dtype, int map, int op) {
    if (dtype == KS_BF16 && map == KS_MAP_WIDEN_F32) return half_entry<BF16Bits>(op);
    if (dtype == KS_F16 && map == KS_MAP_WIDEN_F32) return half_entry<F16Bits>(op);
    if (dtype != KS_U8 || op != KS_SUM) return nullptr;
    if (map == KS_MAP_UNIT_FLOAT8) return ReducePair<uint8_t, MappedOp<SumOp<float>, UnitFloat8Map>>::entry();
    if (map == KS_MAP_WIDEN64) return ReducePair<uint8_t, MappedOp<ByteWideSumOp, Widen64Map>>::entry();
    if (map == KS_MAP_IDENTITY) return ReducePair<uint8_t, ByteSumOp>::entry();
    return nullptr;
}
}  // namespace ks
