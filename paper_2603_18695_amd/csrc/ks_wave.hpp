// Wave64 building blocks: cross-lane moves on 32-bit words through DPP, and an
// order-preserving inclusive scan over the 64 lanes built from them.
//
// Paper Sec. IV-A: shuffles are defined for one 32-bit primitive and every
// composite element is moved field by field.  Here the moves are gfx9-family
// DPP modifiers (row shifts inside a row of 16 lanes, then row broadcasts), so
// no LDS and no ds_bpermute is involved.  All callers run with all 64 lanes
// active.
#pragma once

#include "ks_types.hpp"

namespace ks {

constexpr int kWave = 64;

// DPP control encodings (gfx9 family)
constexpr int kDppRowShr1 = 0x111;
constexpr int kDppRowShr2 = 0x112;
constexpr int kDppRowShr4 = 0x114;
constexpr int kDppRowShr8 = 0x118;
constexpr int kDppWaveShr1 = 0x138;   // every lane reads lane-1; lane 0 keeps `old`
constexpr int kDppRowBcast15 = 0x142; // lane 15 of each row -> every lane of the next row
constexpr int kDppRowBcast31 = 0x143; // lane 31 -> every lane of rows 2 and 3

// Move x across lanes according to CTRL.  Lanes without a valid source, and
// lanes in rows not selected by ROW_MASK, receive `fill` instead.
template <int CTRL, int ROW_MASK, class T>
__device__ __forceinline__ T dpp_move(const T &x, const T &fill) {
    auto xs = to_words(x);
    auto fs = to_words(fill);
    typename WordsOf<T>::type r;
#pragma unroll
    for (int k = 0; k < WordsOf<T>::W; ++k)
        r.w[k] = (uint32_t)__builtin_amdgcn_update_dpp((int)fs.w[k], (int)xs.w[k], CTRL, ROW_MASK, 0xf, false);
    return from_words<T>(r);
}

// Value held by `lane` (compile-time or wave-uniform), broadcast to all lanes.
template <class T>
__device__ __forceinline__ T read_lane(const T &x, int lane) {
    auto xs = to_words(x);
    typename WordsOf<T>::type r;
#pragma unroll
    for (int k = 0; k < WordsOf<T>::W; ++k)
        r.w[k] = (uint32_t)__builtin_amdgcn_readlane((int)xs.w[k], lane);
    return from_words<T>(r);
}

// Inclusive scan over the wave in lane order: lane l ends with
// x[0] op x[1] op ... op x[l].  Values arriving from lower lanes are always the
// left operand.  Lanes with nothing to receive combine with the identity.
template <class T, class Op>
__device__ __forceinline__ T wave_inclusive_scan(T x, Op op) {
    const T id = Op::identity();
    x = op(dpp_move<kDppRowShr1, 0xf>(x, id), x);
    x = op(dpp_move<kDppRowShr2, 0xf>(x, id), x);
    x = op(dpp_move<kDppRowShr4, 0xf>(x, id), x);
    x = op(dpp_move<kDppRowShr8, 0xf>(x, id), x);
    x = op(dpp_move<kDppRowBcast15, 0xa>(x, id), x);   // rows 1 and 3 take the total of the row below
    x = op(dpp_move<kDppRowBcast31, 0xc>(x, id), x);   // rows 2 and 3 take the total of lanes 0..31
    return x;
}

// Lane l receives the value of lane l-1; lane 0 receives `fill`.
template <class T>
__device__ __forceinline__ T wave_shift_up(const T &x, const T &fill) {
    return dpp_move<kDppWaveShr1, 0xf>(x, fill);
}

}  // namespace ks
