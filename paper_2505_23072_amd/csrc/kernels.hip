// gfx950 kernels that turn raw safetensors bytes in HBM into typed, aligned tensors (paper
// Section III-B: alignment fix and type conversion done in one pass on the GPU; one rank's
// partition is taken in the same pass).  Pure data movement: HBM-bound, no matrix cores.
//
// Work is a table of pieces (DevDesc).  One workgroup of 1024 threads = 16 wavefronts takes one
// tile of a piece; the piece is found through a hint table (one entry per HINT_SPAN tiles) with
// scalar loads, since it only depends on the workgroup index.  In the vector and spliced paths a
// lane moves one chunk: 16 source bytes when nothing is converted, 8 elements otherwise, always
// written with full 16-byte stores to a 16-byte aligned destination.  Latency is covered by
// occupancy (two workgroups = 32 wavefronts per CU), not by several loads per lane.
//
// The source may start at any byte.  Sources that are a multiple of 4 are read with 4-byte
// aligned 16-byte loads.  Others read the enclosing aligned dwords (one more than the chunk
// holds) and shift them into place with v_alignbyte_b32, so every load stays dword aligned and
// no byte outside the dwords that hold requested bytes is touched.
#include <hip/hip_runtime.h>

#include <cstddef>

#include "fst_internal.h"

namespace fst {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));      // 16 bytes at a 4-byte aligned address
// Everything the kernels touch is global memory; saying so keeps the compiler from emitting flat
// (generic address space) accesses for pointers it cannot trace back to a kernel argument.
#define FST_GLOBAL __attribute__((address_space(1)))

__device__ __forceinline__ u32x4 gload16(const void *p)
{
    return *(const FST_GLOBAL u32x4_a4 *)(p);
}
// The raw bytes are read once and the outputs are not read back: streaming (non-temporal)
// accesses keep them from displacing each other in the caches.
__device__ __forceinline__ u32x4 gload16_stream(const void *p)
{
    return __builtin_nontemporal_load((const FST_GLOBAL u32x4_a4 *)(p));
}
__device__ __forceinline__ uint32_t gload4(const void *p)
{
    return *(const FST_GLOBAL uint32_t *)(p);
}
__device__ __forceinline__ void gstore16(void *p, u32x4 v)
{
    __builtin_nontemporal_store(v, (FST_GLOBAL u32x4 *)(p));
}

struct Chunk32 { u32x4 lo, hi; };                        // up to 32 source or result bytes

__device__ __forceinline__ uint32_t shift_bytes(uint32_t hi, uint32_t lo, uint32_t sh)
{
    return __builtin_amdgcn_alignbyte(hi, lo, sh);       // ({hi,lo} >> 8*sh)[31:0], sh in 0..3
}

// 16 bytes from any address (BYTE) or from a 4-byte aligned one.
template <bool BYTE>
__device__ __forceinline__ u32x4 load16(const uint8_t *src)
{
    if (!BYTE) return gload16_stream(src);
    const uintptr_t a = reinterpret_cast<uintptr_t>(src);
    const uint32_t sh = uint32_t(a) & 3u;
    const uint8_t *p = reinterpret_cast<const uint8_t *>(a & ~uintptr_t(3));
    const u32x4 v = gload16(p);
    const uint32_t e = sh ? gload4(p + 16) : 0u;         // the fifth dword only if it holds wanted bytes
    u32x4 r;
    r.x = shift_bytes(v.y, v.x, sh);
    r.y = shift_bytes(v.z, v.y, sh);
    r.z = shift_bytes(v.w, v.z, sh);
    r.w = shift_bytes(e, v.w, sh);
    return r;
}

template <bool BYTE>
__device__ __forceinline__ Chunk32 load32(const uint8_t *src)
{
    Chunk32 c;
    if (!BYTE) {
        c.lo = gload16_stream(src);
        c.hi = gload16_stream(src + 16);
        return c;
    }
    const uintptr_t a = reinterpret_cast<uintptr_t>(src);
    const uint32_t sh = uint32_t(a) & 3u;
    const uint8_t *p = reinterpret_cast<const uint8_t *>(a & ~uintptr_t(3));
    const u32x4 v = gload16(p);
    const u32x4 w = gload16(p + 16);
    const uint32_t e = sh ? gload4(p + 32) : 0u;
    c.lo.x = shift_bytes(v.y, v.x, sh);
    c.lo.y = shift_bytes(v.z, v.y, sh);
    c.lo.z = shift_bytes(v.w, v.z, sh);
    c.lo.w = shift_bytes(w.x, v.w, sh);
    c.hi.x = shift_bytes(w.y, w.x, sh);
    c.hi.y = shift_bytes(w.z, w.y, sh);
    c.hi.z = shift_bytes(w.w, w.z, sh);
    c.hi.w = shift_bytes(e, w.w, sh);
    return c;
}

// ---- element conversions on bit patterns: round to nearest even, overflow to infinity, gradual
// underflow, sign of zero kept; NaN keeps sign and leading payload bits and is made quiet.

// binary16 -> binary32 (exact).  Subnormals: the 10-bit field m stands for m * 2^-24, which the
// int->float conversion and one exact multiplication produce without a normalisation loop.
__device__ __forceinline__ uint32_t half_to_float(uint32_t h)
{
    const uint32_t sign = (h & 0x8000u) << 16;
    const uint32_t mag = h & 0x7FFFu;
    uint32_t r = (mag << 13) + 0x38000000u;                              // normal: rebias 15 -> 127
    if (mag < 0x0400u) r = __float_as_uint(float(mag) * 0x1p-24f);       // zero and subnormals
    if (mag >= 0x7C00u) r = (mag << 13) | 0x7F800000u | ((mag & 0x3FFu) ? 0x00400000u : 0u);
    return sign | r;
}

// bfloat16 -> binary32: the same bits, 16 places up.
__device__ __forceinline__ uint32_t bfloat_to_float(uint32_t b)
{
    const uint32_t r = b << 16;
    return ((r & 0x7FFFFFFFu) > 0x7F800000u) ? (r | 0x00400000u) : r;
}

// binary32 -> bfloat16: add half an ulp of the result (minus one when the kept lsb is even) and
// truncate; the carry out of the mantissa moves the exponent up, through to infinity.
__device__ __forceinline__ uint32_t float_to_bfloat(uint32_t x)
{
    const uint32_t rounded = (x + 0x7FFFu + ((x >> 16) & 1u)) >> 16;
    const uint32_t nan = (x >> 16) | 0x0040u;
    return ((x & 0x7FFFFFFFu) > 0x7F800000u) ? nan : rounded;
}

// binary32 -> binary16.
__device__ __forceinline__ uint32_t float_to_half(uint32_t x)
{
    const uint32_t sign = (x >> 16) & 0x8000u;
    const uint32_t mag = x & 0x7FFFFFFFu;
    uint32_t r;
    if (mag >= 0x38800000u) {
        // normal result: rebias, round the 13 dropped bits, clamp everything from 65520 up to inf
        const uint32_t t = mag - 0x38000000u;
        r = (t + 0x0FFFu + ((t >> 13) & 1u)) >> 13;
        if (mag >= 0x477FF000u) r = 0x7C00u;
        if (mag > 0x7F800000u) r = 0x7E00u | ((mag >> 13) & 0x1FFu);
    } else {
        // |x| < 2^-14: adding 0.5 lines the value up so that the sum's low mantissa bits are
        // x / 2^-24 rounded to nearest even by the adder itself (ulp of [0.5, 1) is 2^-24)
        r = __float_as_uint(__uint_as_float(mag) + 0.5f) - 0x3F000000u;
    }
    return sign | r;
}

// binary32 -> binary64 (exact).  Subnormals: the 23-bit field m stands for m * 2^-149; the
// integer is exact in binary64 and so is the scaling by a power of two.
__device__ __forceinline__ uint64_t float_to_double(uint32_t x)
{
    const uint64_t sign = uint64_t(x >> 31) << 63;
    const uint32_t mag = x & 0x7FFFFFFFu;
    uint64_t r = (uint64_t(mag) << 29) + 0x3800000000000000ull;         // normal: rebias 127 -> 1023
    if (mag < 0x00800000u) r = uint64_t(__double_as_longlong(double(mag) * 0x1p-149));
    if (mag >= 0x7F800000u)
        r = (uint64_t(mag) << 29) | 0x7FF0000000000000ull | ((mag & 0x7FFFFFu) ? 0x0008000000000000ull : 0ull);
    return sign | r;
}

// binary64 -> binary32.
__device__ __forceinline__ uint32_t double_to_float(uint64_t x)
{
    const uint32_t sign = uint32_t(x >> 32) & 0x80000000u;
    const uint64_t mag = x & 0x7FFFFFFFFFFFFFFFull;
    uint32_t r;
    if (mag > 0x7FF0000000000000ull) {
        r = 0x7FC00000u | uint32_t((mag >> 29) & 0x3FFFFFu);                   // NaN: quiet, leading payload kept
    } else if (mag >= 0x47F0000000000000ull) {
        r = 0x7F800000u;                                                        // 2^128 and above (and infinity)
    } else if (mag >= 0x3810000000000000ull) {
        // normal result: rebias, round the 29 dropped bits; a carry may reach infinity
        const uint64_t t = mag - 0x3800000000000000ull;
        r = uint32_t((t + 0x0FFFFFFFull + ((t >> 29) & 1ull)) >> 29);
    } else {
        // |x| < 2^-126: adding 2^-97 lines the value up so that the sum's low mantissa bits are
        // |x| / 2^-149 rounded to nearest even by the adder itself (ulp of [2^-97, 2^-96) is 2^-149)
        r = uint32_t(uint64_t(__double_as_longlong(__longlong_as_double((long long)mag) + 0x1p-97)) - 0x39E0000000000000ull);
    }
    return sign | r;
}

template <uint32_t CONV> struct ConvTraits;
// SRC / DST: bytes of one chunk before and after; UNITS: units per chunk (bytes when copying).
template <> struct ConvTraits<CONV_COPY> { static constexpr uint32_t SRC = 16, DST = 16, UNITS = 16; };
template <> struct ConvTraits<CONV_H2B> { static constexpr uint32_t SRC = 16, DST = 16, UNITS = 8; };
template <> struct ConvTraits<CONV_B2H> { static constexpr uint32_t SRC = 16, DST = 16, UNITS = 8; };
template <> struct ConvTraits<CONV_H2F> { static constexpr uint32_t SRC = 16, DST = 32, UNITS = 8; };
template <> struct ConvTraits<CONV_B2F> { static constexpr uint32_t SRC = 16, DST = 32, UNITS = 8; };
template <> struct ConvTraits<CONV_F2H> { static constexpr uint32_t SRC = 32, DST = 16, UNITS = 8; };
template <> struct ConvTraits<CONV_F2B> { static constexpr uint32_t SRC = 32, DST = 16, UNITS = 8; };
template <> struct ConvTraits<CONV_D2F> { static constexpr uint32_t SRC = 32, DST = 16, UNITS = 4; };
template <> struct ConvTraits<CONV_F2D> { static constexpr uint32_t SRC = 16, DST = 32, UNITS = 4; };

template <uint32_t CONV>
__device__ __forceinline__ uint32_t convert_bits(uint32_t v)
{
    if (CONV == CONV_H2B) return float_to_bfloat(half_to_float(v));     // one rounding: widening is exact
    if (CONV == CONV_B2H) return float_to_half(bfloat_to_float(v));
    if (CONV == CONV_H2F) return half_to_float(v);
    if (CONV == CONV_B2F) return bfloat_to_float(v);
    if (CONV == CONV_F2H) return float_to_half(v);
    if (CONV == CONV_F2B) return float_to_bfloat(v);
    return v;
}

// One element of any width (the element path).
template <uint32_t CONV>
__device__ __forceinline__ uint64_t convert_element(uint64_t v)
{
    if (CONV == CONV_D2F) return double_to_float(v);
    if (CONV == CONV_F2D) return float_to_double(uint32_t(v));
    return convert_bits<CONV>(uint32_t(v));
}

template <uint32_t CONV>
__device__ __forceinline__ uint32_t narrow_pair(uint32_t packed)       // two 16-bit -> two 16-bit
{
    return convert_bits<CONV>(packed & 0xFFFFu) | (convert_bits<CONV>(packed >> 16) << 16);
}

// ---- the same conversions on the conversion instructions of the vector ALU, for chunks without
// infinities and NaNs.  For every other input IEEE 754 fixes the result of a round-to-nearest-even
// conversion bit for bit, and the kernels run with denormals kept and that rounding mode (the
// defaults of a HIP kernel), so both formulations agree there; the parity tests compare them over
// all 16-bit inputs and all 2^32 binary32 inputs.  NaN payload handling is a matter of choice, so
// chunks that hold an all-ones exponent take the integer formulation above.
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ f32x2 widen_half_pair(uint32_t w)
{
    return __builtin_convertvector(__builtin_bit_cast(f16x2, w), f32x2);
}
__device__ __forceinline__ f32x2 widen_bfloat_pair(uint32_t w)
{
    f32x2 f;
    f.x = __uint_as_float(w << 16);
    f.y = __uint_as_float(w & 0xFFFF0000u);
    return f;
}
__device__ __forceinline__ f32x2 float_pair(uint32_t a, uint32_t b)
{
    f32x2 f;
    f.x = __uint_as_float(a);
    f.y = __uint_as_float(b);
    return f;
}
__device__ __forceinline__ double double_of(uint32_t lo, uint32_t hi)
{
    return __longlong_as_double((long long)(uint64_t(lo) | (uint64_t(hi) << 32)));
}
__device__ __forceinline__ uint32_t narrow_to_bfloat_pair(f32x2 f)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
__device__ __forceinline__ uint32_t narrow_to_half_pair(f32x2 f)
{
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2));
}

// True when some element of the chunk has an all-ones exponent field.  Adding the field's lowest
// bit to the masked field carries into the bit above it exactly when the field is all ones; for
// two 16-bit elements in a word the lower carry stops at bit 15, below the upper element.
template <uint32_t CONV>
__device__ __forceinline__ bool chunk_has_inf_or_nan(const Chunk32 &in)
{
    if (CONV == CONV_D2F) {
        // the exponent of a binary64 element sits in its upper word
        constexpr uint32_t MASK = 0x7FF00000u, LOW = 0x00100000u;
        const uint32_t acc = ((in.lo.y & MASK) + LOW) | ((in.lo.w & MASK) + LOW) | ((in.hi.y & MASK) + LOW) |
                             ((in.hi.w & MASK) + LOW);
        return (acc & 0x80000000u) != 0;
    }
    constexpr bool WIDE = CONV == CONV_F2H || CONV == CONV_F2B || CONV == CONV_F2D;
    constexpr uint32_t MASK = WIDE ? 0x7F800000u : CONV == CONV_B2H ? 0x7F807F80u : 0x7C007C00u;
    constexpr uint32_t LOW = WIDE ? 0x00800000u : CONV == CONV_B2H ? 0x00800080u : 0x04000400u;
    uint32_t acc = ((in.lo.x & MASK) + LOW) | ((in.lo.y & MASK) + LOW) | ((in.lo.z & MASK) + LOW) |
                   ((in.lo.w & MASK) + LOW);
    if (ConvTraits<CONV>::SRC == 32)
        acc |= ((in.hi.x & MASK) + LOW) | ((in.hi.y & MASK) + LOW) | ((in.hi.z & MASK) + LOW) |
               ((in.hi.w & MASK) + LOW);
    return (acc & 0x80008000u) != 0;
}

template <uint32_t CONV>
__device__ __forceinline__ Chunk32 convert_chunk_finite(const Chunk32 &in)
{
    Chunk32 o;
    if (CONV == CONV_H2B) {
        o.lo.x = narrow_to_bfloat_pair(widen_half_pair(in.lo.x));
        o.lo.y = narrow_to_bfloat_pair(widen_half_pair(in.lo.y));
        o.lo.z = narrow_to_bfloat_pair(widen_half_pair(in.lo.z));
        o.lo.w = narrow_to_bfloat_pair(widen_half_pair(in.lo.w));
    } else if (CONV == CONV_B2H) {
        o.lo.x = narrow_to_half_pair(widen_bfloat_pair(in.lo.x));
        o.lo.y = narrow_to_half_pair(widen_bfloat_pair(in.lo.y));
        o.lo.z = narrow_to_half_pair(widen_bfloat_pair(in.lo.z));
        o.lo.w = narrow_to_half_pair(widen_bfloat_pair(in.lo.w));
    } else if (CONV == CONV_H2F) {
        const f32x2 a = widen_half_pair(in.lo.x), b = widen_half_pair(in.lo.y);
        const f32x2 c = widen_half_pair(in.lo.z), d = widen_half_pair(in.lo.w);
        o.lo.x = __float_as_uint(a.x); o.lo.y = __float_as_uint(a.y);
        o.lo.z = __float_as_uint(b.x); o.lo.w = __float_as_uint(b.y);
        o.hi.x = __float_as_uint(c.x); o.hi.y = __float_as_uint(c.y);
        o.hi.z = __float_as_uint(d.x); o.hi.w = __float_as_uint(d.y);
    } else if (CONV == CONV_F2H) {
        o.lo.x = narrow_to_half_pair(float_pair(in.lo.x, in.lo.y));
        o.lo.y = narrow_to_half_pair(float_pair(in.lo.z, in.lo.w));
        o.lo.z = narrow_to_half_pair(float_pair(in.hi.x, in.hi.y));
        o.lo.w = narrow_to_half_pair(float_pair(in.hi.z, in.hi.w));
    } else if (CONV == CONV_F2B) {
        o.lo.x = narrow_to_bfloat_pair(float_pair(in.lo.x, in.lo.y));
        o.lo.y = narrow_to_bfloat_pair(float_pair(in.lo.z, in.lo.w));
        o.lo.z = narrow_to_bfloat_pair(float_pair(in.hi.x, in.hi.y));
        o.lo.w = narrow_to_bfloat_pair(float_pair(in.hi.z, in.hi.w));
    } else if (CONV == CONV_D2F) {
        o.lo.x = __float_as_uint(float(double_of(in.lo.x, in.lo.y)));
        o.lo.y = __float_as_uint(float(double_of(in.lo.z, in.lo.w)));
        o.lo.z = __float_as_uint(float(double_of(in.hi.x, in.hi.y)));
        o.lo.w = __float_as_uint(float(double_of(in.hi.z, in.hi.w)));
    } else if (CONV == CONV_F2D) {
        const uint64_t a = uint64_t(__double_as_longlong(double(__uint_as_float(in.lo.x))));
        const uint64_t b = uint64_t(__double_as_longlong(double(__uint_as_float(in.lo.y))));
        const uint64_t c = uint64_t(__double_as_longlong(double(__uint_as_float(in.lo.z))));
        const uint64_t d = uint64_t(__double_as_longlong(double(__uint_as_float(in.lo.w))));
        o.lo.x = uint32_t(a); o.lo.y = uint32_t(a >> 32); o.lo.z = uint32_t(b); o.lo.w = uint32_t(b >> 32);
        o.hi.x = uint32_t(c); o.hi.y = uint32_t(c >> 32); o.hi.z = uint32_t(d); o.hi.w = uint32_t(d >> 32);
    }
    return o;
}

// One chunk: 8 elements (or 16 raw bytes) in, converted out.
template <uint32_t CONV>
__device__ __forceinline__ Chunk32 convert_chunk(const Chunk32 &in)
{
    // bfloat16 -> binary32 is a shift either way
    if (CONV != CONV_COPY && CONV != CONV_B2F)
        if (!chunk_has_inf_or_nan<CONV>(in)) return convert_chunk_finite<CONV>(in);
    Chunk32 o;
    if (CONV == CONV_COPY) {
        o.lo = in.lo;
    } else if (CONV == CONV_H2B || CONV == CONV_B2H) {
        o.lo.x = narrow_pair<CONV>(in.lo.x);
        o.lo.y = narrow_pair<CONV>(in.lo.y);
        o.lo.z = narrow_pair<CONV>(in.lo.z);
        o.lo.w = narrow_pair<CONV>(in.lo.w);
    } else if (CONV == CONV_H2F || CONV == CONV_B2F) {
        o.lo.x = convert_bits<CONV>(in.lo.x & 0xFFFFu);
        o.lo.y = convert_bits<CONV>(in.lo.x >> 16);
        o.lo.z = convert_bits<CONV>(in.lo.y & 0xFFFFu);
        o.lo.w = convert_bits<CONV>(in.lo.y >> 16);
        o.hi.x = convert_bits<CONV>(in.lo.z & 0xFFFFu);
        o.hi.y = convert_bits<CONV>(in.lo.z >> 16);
        o.hi.z = convert_bits<CONV>(in.lo.w & 0xFFFFu);
        o.hi.w = convert_bits<CONV>(in.lo.w >> 16);
    } else if (CONV == CONV_D2F) {
        o.lo.x = double_to_float(in.lo.x | (uint64_t(in.lo.y) << 32));
        o.lo.y = double_to_float(in.lo.z | (uint64_t(in.lo.w) << 32));
        o.lo.z = double_to_float(in.hi.x | (uint64_t(in.hi.y) << 32));
        o.lo.w = double_to_float(in.hi.z | (uint64_t(in.hi.w) << 32));
    } else if (CONV == CONV_F2D) {
        const uint64_t a = float_to_double(in.lo.x), b = float_to_double(in.lo.y);
        const uint64_t c = float_to_double(in.lo.z), d = float_to_double(in.lo.w);
        o.lo.x = uint32_t(a); o.lo.y = uint32_t(a >> 32); o.lo.z = uint32_t(b); o.lo.w = uint32_t(b >> 32);
        o.hi.x = uint32_t(c); o.hi.y = uint32_t(c >> 32); o.hi.z = uint32_t(d); o.hi.w = uint32_t(d >> 32);
    } else {
        o.lo.x = convert_bits<CONV>(in.lo.x) | (convert_bits<CONV>(in.lo.y) << 16);
        o.lo.y = convert_bits<CONV>(in.lo.z) | (convert_bits<CONV>(in.lo.w) << 16);
        o.lo.z = convert_bits<CONV>(in.hi.x) | (convert_bits<CONV>(in.hi.y) << 16);
        o.lo.w = convert_bits<CONV>(in.hi.z) | (convert_bits<CONV>(in.hi.w) << 16);
    }
    return o;
}

// A piece's table entry in scalar registers.  The entry is fetched with one 64-byte scalar load:
// field-by-field loads would each wait for the one before, and that chain is the longest part of
// a wavefront's life before its own load is in flight.
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
struct PieceRegs {
    u32x16 w;
    __device__ __forceinline__ uint64_t src_off() const { return w[0] | (uint64_t(w[1]) << 32); }
    __device__ __forceinline__ uint64_t src_stride() const { return w[2] | (uint64_t(w[3]) << 32); }
    __device__ __forceinline__ uint64_t dst() const { return w[4] | (uint64_t(w[5]) << 32); }
    __device__ __forceinline__ uint64_t n_units() const { return w[6] | (uint64_t(w[7]) << 32); }
    __device__ __forceinline__ uint32_t units_per_row() const { return w[8]; }
    __device__ __forceinline__ uint32_t tile0() const { return w[9]; }
    __device__ __forceinline__ uint32_t n_tiles() const { return w[10]; }
    __device__ __forceinline__ uint32_t div_m() const { return w[11]; }
    __device__ __forceinline__ uint32_t div_s() const { return w[12]; }
};
static_assert(offsetof(DevDesc, src_off) == 0 && offsetof(DevDesc, src_stride) == 8 && offsetof(DevDesc, dst) == 16 &&
              offsetof(DevDesc, n_units) == 24 && offsetof(DevDesc, units_per_row) == 32 &&
              offsetof(DevDesc, tile0) == 36 && offsetof(DevDesc, n_tiles) == 40 && offsetof(DevDesc, div_m) == 44 &&
              offsetof(DevDesc, div_s) == 48, "PieceRegs reads DevDesc by dword position");

// The piece that owns tile `b`.  hints[k] names the piece that holds tile k*HINT_SPAN (the last
// piece for the entry past the end), so the owner lies between hints[b/HINT_SPAN] and the next
// entry: for a large tensor the two are equal and nothing is searched; a span full of small
// tensors costs a binary search over first-tile fields, at most log2(HINT_SPAN) steps.
__device__ __forceinline__ PieceRegs find_piece(const DevDesc *__restrict__ descs,
                                                const uint32_t *__restrict__ hints, uint32_t b)
{
    uint32_t lo = hints[b / HINT_SPAN], hi = hints[b / HINT_SPAN + 1];
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (descs[mid].tile0 <= b) lo = mid; else hi = mid - 1;
    }
    PieceRegs p;
    p.w = *reinterpret_cast<const u32x16 *>(descs + lo);
    return p;
}

// n / d for n < 2^31 with the multiplier the host derived from d (see division_magic).
__device__ __forceinline__ uint32_t fast_div(uint32_t n, uint32_t m, uint32_t s)
{
    return __umulhi(n << 1, m) >> s;
}

// One chunk per lane: chunk c of the piece (c < n_units) is read at its row/column offset from
// `src` and written at dst + c*CD.
template <uint32_t CONV, bool BYTE>
__device__ __forceinline__ void vec_chunk(const uint8_t *src, uint8_t *dst, uint32_t c, const PieceRegs &d)
{
    constexpr uint32_t CS = ConvTraits<CONV>::SRC, CD = ConvTraits<CONV>::DST;
    const uint32_t upr = d.units_per_row();
    const uint8_t *s;
    if (upr == 0) {
        s = src + uint64_t(c) * CS;                                  // one row of any length
    } else {
        const uint32_t r = fast_div(c, d.div_m(), d.div_s());
        s = src + uint64_t(r) * d.src_stride() + uint64_t(c - r * upr) * CS;
    }
    Chunk32 v;
    if (CS == 16) v.lo = load16<BYTE>(s); else v = load32<BYTE>(s);
    const Chunk32 o = convert_chunk<CONV>(v);
    uint8_t *t = dst + uint64_t(c) * CD;
    gstore16(t, o.lo);
    if (CD == 32) gstore16(t + 16, o.hi);
}

template <uint32_t CONV, bool BYTE>
__global__ __launch_bounds__(VEC_BLOCK_THREADS) void materialize_vec(const DevDesc *__restrict__ descs,
                                                                     const uint32_t *__restrict__ hints,
                                                                     const uint8_t *__restrict__ raw,
                                                                     uint32_t tile_base)
{
    const uint32_t b = tile_base + tile_of_workgroup(blockIdx.x, gridDim.x);
    const PieceRegs d = find_piece(descs, hints, b);
    const uint32_t t = b - d.tile0();                                   // tile inside the piece
    const uint32_t c0 = t * VEC_TILE_UNITS;                             // a piece has at most 2^31 chunks
    // only a piece's last tile can be short; decided on 32-bit tile counts
    const uint32_t n = (t + 1 == d.n_tiles()) ? uint32_t(d.n_units()) - c0 : VEC_TILE_UNITS;
    if (threadIdx.x < n)
        vec_chunk<CONV, BYTE>(raw + d.src_off(), reinterpret_cast<uint8_t *>(d.dst()), c0 + threadIdx.x, d);
}

// Bytes [0, kb) of `a` followed by bytes [kb, ...) of `b`, word by word (kb in 1 .. size-1).
__device__ __forceinline__ uint32_t splice_word(uint32_t a, uint32_t b, int32_t kb, int32_t word)
{
    const int32_t t = kb - 4 * word;                   // bytes of this word that come from `a`
    const uint32_t m = t <= 0 ? 0u : t >= 4 ? 0xFFFFFFFFu : (1u << (8 * t)) - 1u;
    return (a & m) | (b & ~m);
}
template <uint32_t CS>
__device__ __forceinline__ Chunk32 splice_chunk(const Chunk32 &a, const Chunk32 &b, uint32_t kb)
{
    Chunk32 o;
    const int32_t k = int32_t(kb);
    o.lo.x = splice_word(a.lo.x, b.lo.x, k, 0);
    o.lo.y = splice_word(a.lo.y, b.lo.y, k, 1);
    o.lo.z = splice_word(a.lo.z, b.lo.z, k, 2);
    o.lo.w = splice_word(a.lo.w, b.lo.w, k, 3);
    if (CS == 32) {
        o.hi.x = splice_word(a.hi.x, b.hi.x, k, 4);
        o.hi.y = splice_word(a.hi.y, b.hi.y, k, 5);
        o.hi.z = splice_word(a.hi.z, b.hi.z, k, 6);
        o.hi.w = splice_word(a.hi.w, b.hi.w, k, 7);
    }
    return o;
}

// Spliced path: rows that are not a whole number of chunks (a dim-1 share whose row segment is,
// say, 2050 bytes).  The output is one contiguous stream; a lane owns one 16-byte aligned chunk of
// it, i.e. CH consecutive units (bytes when copying, elements when converting).  Most chunks lie
// inside one row and are read like a byte-aligned vector chunk.  A chunk that straddles a row end
// takes its first k units from the end of row r and the rest from the start of row r+1: the second
// read starts k units *before* row r+1 (inside row r's stride, since a row has at least CH units),
// so that both reads hold their units at the chunk's own positions and a byte mask splices them.
template <uint32_t CONV>
__global__ __launch_bounds__(VEC_BLOCK_THREADS) void materialize_splice(const DevDesc *__restrict__ descs,
                                                                        const uint32_t *__restrict__ hints,
                                                                        const uint8_t *__restrict__ raw,
                                                                        uint32_t tile_base)
{
    constexpr uint32_t CS = ConvTraits<CONV>::SRC, CD = ConvTraits<CONV>::DST;
    constexpr uint32_t CH = ConvTraits<CONV>::UNITS;                    // units per chunk
    constexpr uint32_t US = CS / CH;                                    // source bytes per unit
    const uint32_t b = tile_base + tile_of_workgroup(blockIdx.x, gridDim.x);
    const PieceRegs d = find_piece(descs, hints, b);
    const uint32_t t = b - d.tile0();
    const uint32_t c0 = t * VEC_TILE_UNITS;
    const uint32_t n = (t + 1 == d.n_tiles()) ? uint32_t(d.n_units()) - c0 : VEC_TILE_UNITS;
    if (threadIdx.x >= n) return;
    const uint32_t c = c0 + threadIdx.x;
    const uint32_t u0 = c * CH;                                         // the piece has fewer than 2^31 units
    const uint32_t upr = d.units_per_row();
    const uint32_t r = fast_div(u0, d.div_m(), d.div_s());
    const uint32_t col = u0 - r * upr;
    const uint8_t *row = raw + d.src_off() + uint64_t(r) * d.src_stride();
    Chunk32 v;
    if (CS == 16) v.lo = load16<true>(row + uint64_t(col) * US); else v = load32<true>(row + uint64_t(col) * US);
    const uint32_t k = upr - col;                                       // units left in row r
    if (k < CH) {
        const uint8_t *next = row + d.src_stride() - k * US;
        Chunk32 w;
        if (CS == 16) w.lo = load16<true>(next); else w = load32<true>(next);
        v = splice_chunk<CS>(v, w, k * US);
    }
    const Chunk32 o = convert_chunk<CONV>(v);
    uint8_t *out = reinterpret_cast<uint8_t *>(d.dst()) + uint64_t(c) * CD;
    gstore16(out, o.lo);
    if (CD == 32) gstore16(out + 16, o.hi);
}

// Element path: tails shorter than a chunk, rows shorter than a chunk, and pieces whose first
// output byte is not 16-byte aligned.  One element (one byte when nothing is converted) per thread
// and step; sources are read bytewise; indices are 64-bit.
template <uint32_t CONV>
__global__ __launch_bounds__(ELEM_BLOCK_THREADS) void materialize_elem(const DevDesc *__restrict__ descs,
                                                                       const uint32_t *__restrict__ hints,
                                                                       const uint8_t *__restrict__ raw,
                                                                       uint32_t tile_base)
{
    constexpr uint32_t ES = ConvTraits<CONV>::SRC / ConvTraits<CONV>::UNITS;         // bytes per source element
    constexpr uint32_t ED = ConvTraits<CONV>::DST / ConvTraits<CONV>::UNITS;
    const uint32_t b = tile_base + blockIdx.x;
    const PieceRegs d = find_piece(descs, hints, b);
    const uint32_t t = b - d.tile0();
    const uint64_t e0 = uint64_t(t) * ELEM_TILE_UNITS;
    const uint32_t n = (t + 1 == d.n_tiles()) ? uint32_t(d.n_units() - e0) : ELEM_TILE_UNITS;
    const uint32_t upr = d.units_per_row();
    const uint64_t stride = d.src_stride();
    const uint64_t row0 = e0 / upr;
    const uint32_t col0 = uint32_t(e0 - row0 * upr);
    const uint8_t *src = raw + d.src_off() + row0 * stride;
    uint8_t *dst = reinterpret_cast<uint8_t *>(d.dst()) + e0 * ED;
    for (uint32_t i = threadIdx.x; i < n; i += ELEM_BLOCK_THREADS) {
        const uint64_t cc = uint64_t(col0) + i;
        const uint64_t r = cc / upr;
        const uint8_t *s = src + r * stride + (cc - r * upr) * ES;
        uint64_t v = 0;
#pragma unroll
        for (uint32_t k = 0; k < ES; ++k) v |= uint64_t(*(const FST_GLOBAL uint8_t *)(s + k)) << (8 * k);
        v = convert_element<CONV>(v);
        uint8_t *o = dst + uint64_t(i) * ED;
        if (ED == 1) *(FST_GLOBAL uint8_t *)(o) = uint8_t(v);
        else if (ED == 2) *(FST_GLOBAL uint16_t *)(o) = uint16_t(v);
        else if (ED == 4) *(FST_GLOBAL uint32_t *)(o) = uint32_t(v);
        else *(FST_GLOBAL uint64_t *)(o) = v;
    }
}

template <uint32_t CONV>
int launch_conv(uint32_t variant, const DevDesc *descs, const uint32_t *hints, uint32_t n_tiles, const uint8_t *raw,
                hipStream_t stream)
{
    for (const LaunchPart &part : split_launch(n_tiles)) {
        const dim3 grid(part.n_tiles);
        const uint32_t base = part.tile_base;
        if (variant == 0)
            hipLaunchKernelGGL((materialize_vec<CONV, false>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw, base);
        else if (variant == 1)
            hipLaunchKernelGGL((materialize_vec<CONV, true>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw, base);
        else if (variant == 3)
            hipLaunchKernelGGL((materialize_splice<CONV>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw, base);
        else
            hipLaunchKernelGGL((materialize_elem<CONV>), grid, dim3(ELEM_BLOCK_THREADS), 0, stream, descs, hints, raw, base);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(FST_E_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    }
    return FST_OK;
}

}  // namespace

int launch_class_kernels(uint32_t cls, const DevDesc *descs_dev, const uint32_t *hints_dev, uint32_t n_tiles,
                         const void *raw_dev, void *stream)
{
    if (n_tiles == 0) return FST_OK;
    uint32_t conv, variant;
    if (cls < CONV_COUNT * 2) { conv = cls / 2; variant = cls % 2; }
    else if (cls < CONV_COUNT * 3) { conv = cls - CONV_COUNT * 2; variant = 2; }
    else { conv = cls - CONV_COUNT * 3; variant = 3; }
    const uint8_t *raw = static_cast<const uint8_t *>(raw_dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    switch (conv) {
    case CONV_COPY: return launch_conv<CONV_COPY>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_H2B: return launch_conv<CONV_H2B>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_B2H: return launch_conv<CONV_B2H>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_H2F: return launch_conv<CONV_H2F>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_B2F: return launch_conv<CONV_B2F>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_F2H: return launch_conv<CONV_F2H>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_F2B: return launch_conv<CONV_F2B>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_D2F: return launch_conv<CONV_D2F>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    case CONV_F2D: return launch_conv<CONV_F2D>(variant, descs_dev, hints_dev, n_tiles, raw, s);
    default: return fail(FST_E_ARG, "unknown launch class %u", cls);
    }
}

}  // namespace fst
