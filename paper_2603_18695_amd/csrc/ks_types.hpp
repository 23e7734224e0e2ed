// Element types and operators of the scan library (device side).
//
// An operator is a stateless functor with
//     static constexpr bool commutative;  // may totals be formed in any order? (never assumed otherwise)
//     using acc = ...;                    // type the scan is carried out in
//     static acc identity();              // op(identity, x) == x bit for bit
//     acc operator()(acc l, acc r) const; // l = accumulated (earlier), r = later
//     using chain = ...;                  // optional: a wider operator for everything above one wave's run
// The element type in memory ("io" type) is converted to acc on load and back
// on store (convert<>); for most pairs the two are the same type.  io types are
// trivially copyable and a multiple of 4 bytes: 4, 8 and 16 bytes run in every
// kernel shape, any other size that divides 128 or 144 bytes (12, 24, 32, 36, 48,
// 64, 72 ...) in the blocked arrangement, where a lane holds 8 or 9 consecutive
// 16-byte granules.  acc types are a multiple of 4 bytes and are moved between
// lanes and through memory as arrays of 32-bit words (paper Sec. IV-A: any
// composite type is shuffled field by field as 32-bit pieces).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ks {

template <int W>
struct Words {
    uint32_t w[W];
};

template <class T>
struct WordsOf {
    static_assert(sizeof(T) % 4 == 0, "element size must be a multiple of 4 bytes");
    static constexpr int W = sizeof(T) / 4;
    using type = Words<W>;
};

template <class T>
__device__ __forceinline__ typename WordsOf<T>::type to_words(const T &x) {
    return __builtin_bit_cast(typename WordsOf<T>::type, x);
}
template <class T>
__device__ __forceinline__ T from_words(const typename WordsOf<T>::type &w) {
    return __builtin_bit_cast(T, w);
}

// ---- element structs -------------------------------------------------------

struct AffineF32 {      // the map x -> a*x + b
    float a, b;
};
struct AffineF64 {      // the same map carried in double (accumulation type of AffineF32)
    double a, b;
};
struct ArgmaxI32Cnt64 { // running maximum, where it first occurred, how many seen
    int32_t v;
    int32_t idx;
    int64_t cnt;
};
struct Mat2U32 {        // row-major 2x2 matrix over Z/2^32
    uint32_t m00, m01, m10, m11;
};
struct QuatF32 {
    float w, x, y, z;
};
struct Mat2U64 {        // row-major 2x2 matrix over Z/2^64: a 32-byte element
    uint64_t m00, m01, m10, m11;
};
struct RangeI32Cnt32 {  // smallest and largest value seen and how many: a 12-byte element
    int32_t lo, hi;
    uint32_t cnt;
};

// ---- limits for min / max identities ---------------------------------------

template <class T> struct Limits;
template <> struct Limits<int32_t>  { __device__ static int32_t  lo() { return INT32_MIN; } __device__ static int32_t  hi() { return INT32_MAX; } };
template <> struct Limits<uint32_t> { __device__ static uint32_t lo() { return 0u; }        __device__ static uint32_t hi() { return UINT32_MAX; } };
template <> struct Limits<int64_t>  { __device__ static int64_t  lo() { return INT64_MIN; } __device__ static int64_t  hi() { return INT64_MAX; } };
template <> struct Limits<uint64_t> { __device__ static uint64_t lo() { return 0ull; }      __device__ static uint64_t hi() { return UINT64_MAX; } };
template <> struct Limits<float>    { __device__ static float    lo() { return -__builtin_inff(); } __device__ static float  hi() { return __builtin_inff(); } };
template <> struct Limits<double>   { __device__ static double   lo() { return -__builtin_inf(); }  __device__ static double hi() { return __builtin_inf(); } };

// ---- operators --------------------------------------------------------------

template <class T>
struct SumOp {
    static constexpr bool commutative = true;
    using acc = T;
    __device__ static T identity() { return T(0); }
    __device__ __forceinline__ T operator()(T l, T r) const { return l + r; }
};
// Float32 sums: inside one wave's run (a few thousand neighbouring elements) the additions are
// float32; wave totals, tile aggregates, descriptors and the look-back's running value are double.
// The prefix of a long input is a chain of one addition per tile, and every float32 rounding in
// that chain stays in all later outputs at the magnitude the running sum had when it was made:
// for mixed-sign data the sum comes back to zero with the error of its excursions still in it.
// Carried in double the chain adds nothing; what is left are the roundings inside the runs
// (paper Sec. VII-B validates against a Float64 reference; Sec. V-B leaves the accumulation type open).
template <>
struct SumOp<float> {
    static constexpr bool commutative = true;
    using acc = float;
    using chain = SumOp<double>;
    __device__ static float identity() { return 0.0f; }
    __device__ __forceinline__ float operator()(float l, float r) const { return l + r; }
};
// signed integer sums wrap: add in the unsigned type
template <>
struct SumOp<int32_t> {
    static constexpr bool commutative = true;
    using acc = int32_t;
    __device__ static int32_t identity() { return 0; }
    __device__ __forceinline__ int32_t operator()(int32_t l, int32_t r) const { return (int32_t)((uint32_t)l + (uint32_t)r); }
};
template <>
struct SumOp<int64_t> {
    static constexpr bool commutative = true;
    using acc = int64_t;
    __device__ static int64_t identity() { return 0; }
    __device__ __forceinline__ int64_t operator()(int64_t l, int64_t r) const { return (int64_t)((uint64_t)l + (uint64_t)r); }
};

// Sums over bytes (mapreduce only; the 8-bit types of the paper's mapreduce benchmark, Sec. VII-B).
// A lane adds the bytes of one run in 32 bits (64 bytes of at most 255 each); above the run the
// sum is carried in the chain type: 32 bits when the result is a byte again (the sum modulo 2^8
// is the low byte of any wider wrapped sum), 64 bits when the caller asked for the widened sum.
struct ByteSumOp {
    static constexpr bool commutative = true;
    using acc = uint32_t;
    __device__ static uint32_t identity() { return 0u; }
    __device__ __forceinline__ uint32_t operator()(uint32_t l, uint32_t r) const { return l + r; }
};
struct ByteWideSumOp : ByteSumOp {
    using chain = SumOp<uint64_t>;
};

template <class T>
struct MinOp {
    static constexpr bool commutative = true;
    using acc = T;
    __device__ static T identity() { return Limits<T>::hi(); }
    __device__ __forceinline__ T operator()(T l, T r) const { return r < l ? r : l; }
};
template <class T>
struct MaxOp {
    static constexpr bool commutative = true;
    using acc = T;
    __device__ static T identity() { return Limits<T>::lo(); }
    __device__ __forceinline__ T operator()(T l, T r) const { return r > l ? r : l; }
};

// floating point minimum and maximum: the hardware's own instructions (one instead of a compare and
// a select); with NaN among the inputs the results from there on are unspecified
template <>
struct MinOp<float> {
    static constexpr bool commutative = true;
    using acc = float;
    __device__ static float identity() { return Limits<float>::hi(); }
    __device__ __forceinline__ float operator()(float l, float r) const { return __builtin_fminf(l, r); }
};
template <>
struct MaxOp<float> {
    static constexpr bool commutative = true;
    using acc = float;
    __device__ static float identity() { return Limits<float>::lo(); }
    __device__ __forceinline__ float operator()(float l, float r) const { return __builtin_fmaxf(l, r); }
};
template <>
struct MinOp<double> {
    static constexpr bool commutative = true;
    using acc = double;
    __device__ static double identity() { return Limits<double>::hi(); }
    __device__ __forceinline__ double operator()(double l, double r) const { return __builtin_fmin(l, r); }
};
template <>
struct MaxOp<double> {
    static constexpr bool commutative = true;
    using acc = double;
    __device__ static double identity() { return Limits<double>::lo(); }
    __device__ __forceinline__ double operator()(double l, double r) const { return __builtin_fmax(l, r); }
};

// Apply l first, then r.  Carried in double: the offset b of a long composition
// is a cancelling sum that reaches 1e2..1e3 in magnitude and crosses zero, and
// every later composition multiplies it by a: an a carried in float32 (relative
// error 1e-6 after a thousand factors) then costs 1e-3 absolute, the whole error
// bar.  Tried with float32 inside one wave's run and double only above it: worst
// error 1.2e-3 at n = 5e5, outside the bar.  The float32 inputs and outputs are
// converted at the memory boundary.
struct AffineComposeOp {
    static constexpr bool commutative = false;
    using acc = AffineF64;
    __device__ static AffineF64 identity() { return AffineF64{1.0, 0.0}; }
    __device__ __forceinline__ AffineF64 operator()(AffineF64 l, AffineF64 r) const {
        return AffineF64{r.a * l.a, __builtin_fma(r.a, l.b, r.b)};
    }
};

struct ArgmaxCountOp {
    static constexpr bool commutative = true;   // the better (v, idx) wins whichever side it is on; counts add
    using acc = ArgmaxI32Cnt64;
    __device__ static ArgmaxI32Cnt64 identity() { return ArgmaxI32Cnt64{INT32_MIN, INT32_MAX, 0}; }
    __device__ __forceinline__ ArgmaxI32Cnt64 operator()(ArgmaxI32Cnt64 l, ArgmaxI32Cnt64 r) const {
        const bool take_r = (r.v > l.v) || (r.v == l.v && r.idx < l.idx);
        ArgmaxI32Cnt64 o;
        o.v = take_r ? r.v : l.v;
        o.idx = take_r ? r.idx : l.idx;
        o.cnt = (int64_t)((uint64_t)l.cnt + (uint64_t)r.cnt);
        return o;
    }
};

struct Mat2MulOp {
    static constexpr bool commutative = false;
    using acc = Mat2U32;
    __device__ static Mat2U32 identity() { return Mat2U32{1u, 0u, 0u, 1u}; }
    __device__ __forceinline__ Mat2U32 operator()(Mat2U32 l, Mat2U32 r) const {
        return Mat2U32{l.m00 * r.m00 + l.m01 * r.m10, l.m00 * r.m01 + l.m01 * r.m11,
                       l.m10 * r.m00 + l.m11 * r.m10, l.m10 * r.m01 + l.m11 * r.m11};
    }
};

struct Mat2WideMulOp {
    static constexpr bool commutative = false;
    using acc = Mat2U64;
    __device__ static Mat2U64 identity() { return Mat2U64{1ull, 0ull, 0ull, 1ull}; }
    __device__ __forceinline__ Mat2U64 operator()(Mat2U64 l, Mat2U64 r) const {
        return Mat2U64{l.m00 * r.m00 + l.m01 * r.m10, l.m00 * r.m01 + l.m01 * r.m11,
                       l.m10 * r.m00 + l.m11 * r.m10, l.m10 * r.m01 + l.m11 * r.m11};
    }
};

struct RangeCountOp {
    static constexpr bool commutative = true;
    using acc = RangeI32Cnt32;
    __device__ static RangeI32Cnt32 identity() { return RangeI32Cnt32{INT32_MAX, INT32_MIN, 0u}; }
    __device__ __forceinline__ RangeI32Cnt32 operator()(RangeI32Cnt32 l, RangeI32Cnt32 r) const {
        return RangeI32Cnt32{r.lo < l.lo ? r.lo : l.lo, r.hi > l.hi ? r.hi : l.hi, l.cnt + r.cnt};
    }
};

struct QuatMulOp {   // Hamilton product l * r
    static constexpr bool commutative = false;
    using acc = QuatF32;
    __device__ static QuatF32 identity() { return QuatF32{1.0f, 0.0f, 0.0f, 0.0f}; }
    __device__ __forceinline__ QuatF32 operator()(QuatF32 l, QuatF32 r) const {
        return QuatF32{l.w * r.w - l.x * r.x - l.y * r.y - l.z * r.z,
                       l.w * r.x + l.x * r.w + l.y * r.z - l.z * r.y,
                       l.w * r.y - l.x * r.z + l.y * r.w + l.z * r.x,
                       l.w * r.z + l.x * r.y - l.y * r.x + l.z * r.w};
    }
};

// ---- maps: scan(f, op, src) ----------------------------------------------------
// Paper Sec. IV-A, the high-level interface: out[i] = f(src[0]) op ... op f(src[i]).
// A map is a stateless functor T -> T applied to every element as it is loaded;
// MappedOp<Op, Map> is Op with that map attached, and is what the kernels see.
struct IdentityMap {
    template <class T>
    __device__ __forceinline__ T operator()(const T &x) const { return x; }
};
struct SquareMap {   // x * x; integers wrap
    __device__ __forceinline__ float operator()(float x) const { return x * x; }
    __device__ __forceinline__ double operator()(double x) const { return x * x; }
    __device__ __forceinline__ int32_t operator()(int32_t x) const { return (int32_t)((uint32_t)x * (uint32_t)x); }
    __device__ __forceinline__ uint32_t operator()(uint32_t x) const { return x * x; }
    __device__ __forceinline__ int64_t operator()(int64_t x) const { return (int64_t)((uint64_t)x * (uint64_t)x); }
    __device__ __forceinline__ uint64_t operator()(uint64_t x) const { return x * x; }
};
struct AbsMap {      // |x|; the most negative integer maps to itself (two's complement)
    __device__ __forceinline__ float operator()(float x) const { return __builtin_fabsf(x); }
    __device__ __forceinline__ double operator()(double x) const { return __builtin_fabs(x); }
    __device__ __forceinline__ int32_t operator()(int32_t x) const { return x < 0 ? (int32_t)(0u - (uint32_t)x) : x; }
    __device__ __forceinline__ int64_t operator()(int64_t x) const { return x < 0 ? (int64_t)(0ull - (uint64_t)x) : x; }
};
struct NonzeroMap {  // 1 where x != 0, else 0: a sum scan of it numbers the kept elements of a compaction
    template <class T>
    __device__ __forceinline__ T operator()(const T &x) const { return x != T(0) ? T(1) : T(0); }
};

// 16-bit floats as they lie in memory (reductions only: promoted to float32 as they are loaded).
struct BF16Bits {   // bfloat16: the upper half of a float32
    uint16_t bits;
};
struct F16Bits {    // IEEE binary16
    uint16_t bits;
};

// Maps that change the type, f: T -> S (paper Sec. II-C): `result` is S, the type of what a
// mapreduce with this map writes.
struct WidenF32Map {   // the float32 of the same value: exact for both formats
    using result = float;
    __device__ __forceinline__ float operator()(BF16Bits x) const {
        return __builtin_bit_cast(float, (uint32_t)x.bits << 16);
    }
    __device__ __forceinline__ float operator()(F16Bits x) const {
        return (float)__builtin_bit_cast(_Float16, x.bits);
    }
};
struct Widen64Map {   // a byte as an integer that sums of any length cannot wrap
    using result = uint64_t;
    __device__ __forceinline__ uint32_t operator()(uint8_t c) const { return c; }
};
// Code c = level c of 256 evenly spaced levels from -1 to +1 (paper Sec. VII-B, UnitFloat8),
// (2c - 255) / 255, promoted to float32.  x = 2c - 255 is exact.  One multiplication by the
// float32 nearest to 1/255 would be off by one unit in the last place for half of the codes, so
// 1/255 is carried as two float32 constants, hi + lo, and x * hi + (x * lo) is rounded once by
// the fused operation: the float32 nearest to the rational level for every one of the 256 codes
// (checked code by code against exact rationals).
struct UnitFloat8Map {
    using result = float;
    static constexpr float kHi = 0x1.010102p-8f;     // float32 nearest to 1/255
    static constexpr float kLo = -0x1.fdfdfep-33f;   // float32 nearest to 1/255 - kHi
    __device__ __forceinline__ float operator()(uint8_t c) const {
        const float x = __builtin_fmaf((float)c, 2.0f, -255.0f);
        return __builtin_fmaf(x, kHi, x * kLo);
    }
};

template <class Op, class Map>
struct MappedOp : Op {
    using map = Map;
    using unmapped = Op;
};

template <class Op, class = void>
struct MapOf {
    using type = IdentityMap;
    using unmapped = Op;
    static constexpr bool mapped = false;
};
template <class Op>
struct MapOf<Op, decltype((void)sizeof(typename Op::map))> {
    using type = typename Op::map;
    using unmapped = typename Op::unmapped;
    static constexpr bool mapped = true;
};

// ---- chain type: what is carried above one wave's run ----------------------------
// ChainOf<Op>::op is the operator that combines wave totals, tile aggregates and descriptor values,
// ChainOf<Op>::type its value type; for most operators they are the operator itself (without its
// map) and its acc.  convert<> moves values between acc and the chain type.
template <class Op, class = void>
struct ChainOf {
    using op = typename MapOf<Op>::unmapped;
    using type = typename Op::acc;
};
template <class Op>
struct ChainOf<Op, decltype((void)sizeof(typename Op::chain))> {
    using op = typename Op::chain;
    using type = typename op::acc;
};

// ResultOf<Op, IO>::type: what a mapreduce writes: the map's result type if it names one, else IO.
template <class Op, class IO, class = void>
struct ResultOf {
    using type = IO;
    static constexpr bool from_map = false;
};
template <class Op, class IO>
struct ResultOf<Op, IO, decltype((void)sizeof(typename MapOf<Op>::type::result))> {
    using type = typename MapOf<Op>::type::result;
    static constexpr bool from_map = true;
};

// ---- conversions between memory type, accumulation type and chain type ------------

template <class To, class From>
struct Convert {
    static_assert(sizeof(To) == 0, "no conversion between these element types");
};
template <class T>
struct Convert<T, T> {
    __device__ __forceinline__ static T apply(const T &x) { return x; }
};
template <>
struct Convert<double, float> {
    __device__ __forceinline__ static double apply(const float &x) { return (double)x; }
};
template <>
struct Convert<float, double> {
    __device__ __forceinline__ static float apply(const double &x) { return (float)x; }
};
// float32 -> 16-bit floats: round to nearest, ties to even (what a scan of 16-bit floats stores)
template <>
struct Convert<BF16Bits, float> {
    __device__ __forceinline__ static BF16Bits apply(const float &x) {
        return BF16Bits{__builtin_bit_cast(uint16_t, (__bf16)x)};   // gfx950 converts in hardware, two per instruction
    }
};
template <>
struct Convert<F16Bits, float> {
    __device__ __forceinline__ static F16Bits apply(const float &x) {
        return F16Bits{__builtin_bit_cast(uint16_t, (_Float16)x)};
    }
};
template <>
struct Convert<uint32_t, uint8_t> {
    __device__ __forceinline__ static uint32_t apply(const uint8_t &x) { return x; }
};
template <>
struct Convert<uint8_t, uint32_t> {   // modulo 2^8
    __device__ __forceinline__ static uint8_t apply(const uint32_t &x) { return (uint8_t)x; }
};
template <>
struct Convert<uint64_t, uint32_t> {
    __device__ __forceinline__ static uint64_t apply(const uint32_t &x) { return x; }
};
template <>
struct Convert<AffineF64, AffineF32> {
    __device__ __forceinline__ static AffineF64 apply(const AffineF32 &x) { return AffineF64{(double)x.a, (double)x.b}; }
};
template <>
struct Convert<AffineF32, AffineF64> {
    __device__ __forceinline__ static AffineF32 apply(const AffineF64 &x) { return AffineF32{(float)x.a, (float)x.b}; }
};
template <class To, class From>
__device__ __forceinline__ To convert(const From &x) {
    return Convert<To, From>::apply(x);
}

}  // namespace ks
