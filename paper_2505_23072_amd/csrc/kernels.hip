// gfx950 kernels that turn raw safetensors bytes in HBM into typed, aligned tensors (paper
// Section III-B: alignment fix and type conversion done in one pass on the GPU; one rank's
// partition is taken in the same pass).  Pure data movement: HBM-bound, no matrix cores.
//
// Work is a table of pieces (DevDesc).  A workgroup of 1024 threads = 16 wavefronts takes 16
// consecutive tiles of its launch, one per wavefront (a tile is 64 chunks); the piece a tile
// belongs to is found through a hint table (one entry per HINT_SPAN tiles) with scalar loads,
// since it only depends on the workgroup and wavefront index.  In the vector, spliced and gather
// paths a lane moves one chunk: 16 source bytes when nothing is converted, else 2 to 8 elements
// (see ConvTraits), written with full-width stores to an aligned destination.  Latency is covered
// by occupancy (two workgroups = 32 wavefronts per CU), not by several loads per lane.
//
// The source may start at any byte.  Sources that are a multiple of 4 are read with 4-byte
// aligned 16-byte loads.  Others read the enclosing aligned dwords (one more than the chunk
// holds) and shift them into place with v_alignbyte_b32, so every load stays dword aligned and
// no byte outside the dwords that hold requested bytes is touched.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <utility>

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
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef u32x2 u32x2_a4 __attribute__((aligned(4)));
typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
typedef u32x3 u32x3_a4 __attribute__((aligned(4)));
__device__ __forceinline__ void gstore8(void *p, uint32_t x, uint32_t y)
{
    u32x2 v;
    v.x = x;
    v.y = y;
    __builtin_nontemporal_store(v, (FST_GLOBAL u32x2 *)(p));
}

struct Chunk32 { u32x4 lo, hi; };                        // up to 32 source bytes, up to 16 result bytes (in lo)

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

// 8 bytes (in .x and .y) from any address (BYTE) or from a 4-byte aligned one.  The dword that holds
// the last wanted bytes of an unaligned chunk is fetched only when there is one (the byte offset is
// not 0): either in the same instruction as the others (FUSED: one of two load forms behind a
// branch; best when a wavefront's lanes all have the same offset, as in the vector path: 6.15 against
// 5.7 TB/s on BF16 -> F32) or with a predicated load of its own (no branch; best in the spliced path,
// where the offset changes from row to row: 5.4 against 4.75 TB/s on 2050-byte row segments).
template <bool BYTE, bool FUSED>
__device__ __forceinline__ u32x4 load8(const uint8_t *src)
{
    u32x4 r = {0u, 0u, 0u, 0u};
    if (!BYTE) {
        const u32x2 v = __builtin_nontemporal_load((const FST_GLOBAL u32x2_a4 *)(src));
        r.x = v.x;
        r.y = v.y;
        return r;
    }
    const uintptr_t a = reinterpret_cast<uintptr_t>(src);
    const uint32_t sh = uint32_t(a) & 3u;
    const uint8_t *p = reinterpret_cast<const uint8_t *>(a & ~uintptr_t(3));
    if (!FUSED) {
        const u32x2 v = *(const FST_GLOBAL u32x2_a4 *)(p);
        const uint32_t e = sh ? gload4(p + 8) : 0u;
        r.x = shift_bytes(v.y, v.x, sh);
        r.y = shift_bytes(e, v.y, sh);
    } else if (sh) {
        const u32x3 v = *(const FST_GLOBAL u32x3_a4 *)(p);
        r.x = shift_bytes(v.y, v.x, sh);
        r.y = shift_bytes(v.z, v.y, sh);
    } else {
        const u32x2 v = *(const FST_GLOBAL u32x2_a4 *)(p);
        r.x = v.x;
        r.y = v.y;
    }
    return r;
}

// 4 bytes (in .x) from any address (BYTE) or from a 4-byte aligned one; FUSED as in load8.
template <bool BYTE, bool FUSED>
__device__ __forceinline__ u32x4 load4(const uint8_t *src)
{
    u32x4 r = {0u, 0u, 0u, 0u};
    if (!BYTE) {
        r.x = __builtin_nontemporal_load((const FST_GLOBAL uint32_t *)(src));
        return r;
    }
    const uintptr_t a = reinterpret_cast<uintptr_t>(src);
    const uint32_t sh = uint32_t(a) & 3u;
    const uint8_t *p = reinterpret_cast<const uint8_t *>(a & ~uintptr_t(3));
    if (!FUSED) {
        const uint32_t v = gload4(p);
        const uint32_t e = sh ? gload4(p + 4) : 0u;      // the second dword only if it holds wanted bytes
        r.x = shift_bytes(e, v, sh);
    } else if (sh) {
        const u32x2 v = *(const FST_GLOBAL u32x2_a4 *)(p);
        r.x = shift_bytes(v.y, v.x, sh);
    } else {
        r.x = gload4(p);
    }
    return r;
}

template <bool BYTE>
__device__ __forceinline__ Chunk32 load32(const uint8_t *src)
{
    Chunk32 c;
    if (!BYTE) {
        // two loads per lane share their cache lines with the neighbouring lanes' loads: a streaming
        // hint on the first would let go of lines the second still needs (measured: 6 % slower)
        c.lo = gload16(src);
        c.hi = gload16(src + 16);
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

// binary64 -> binary32 rounded to odd: the binary32 neighbour towards zero, with its lowest bit set
// when the value is not exact.  A second rounding to nearest even into a format at least two bits
// shorter (binary16, bfloat16) then gives what one rounding from binary64 gives: the odd last bit
// keeps an inexact value off every tie and on the right side of it.  NaN goes by the NaN rule.
__device__ __forceinline__ uint32_t double_to_float_odd(uint64_t x)
{
    if ((x & 0x7FFFFFFFFFFFFFFFull) > 0x7FF0000000000000ull) return double_to_float(x);
    const double d = __longlong_as_double((long long)x);
    const float f = float(d);                                   // to nearest even
    uint32_t b = __float_as_uint(f);
    const double back = double(f);
    if (back != d) {                                            // inexact (an overflow to infinity included)
        if (__builtin_fabs(back) > __builtin_fabs(d)) b -= 1u;  // one step towards zero
        b |= 1u;
    }
    return b;
}

// 8-bit E5M2 (1-5-2, bias 15, infinities and NaNs as in IEEE 754) -> binary16: the same layout with
// eight more mantissa bits.
__device__ __forceinline__ uint32_t e5m2_to_half(uint32_t b)
{
    const uint32_t h = b << 8;
    return ((h & 0x7FFFu) > 0x7C00u) ? (h | 0x0200u) : h;
}

// 8-bit E4M3 (1-4-3, bias 7; no infinity, the exponent field's last binade holds ordinary values up
// to 448 and mantissa all ones there is the NaN) -> binary32 (exact).  Subnormals: the 3-bit field m
// stands for m * 2^-9.
__device__ __forceinline__ uint32_t e4m3_to_float(uint32_t b)
{
    const uint32_t sign = (b & 0x80u) << 24;
    const uint32_t mag = b & 0x7Fu;
    uint32_t r = (mag << 20) + 0x3C000000u;                              // normal: rebias 7 -> 127
    if (mag < 0x08u) r = __float_as_uint(float(mag) * 0x1p-9f);          // zero and subnormals
    if (mag == 0x7Fu) r = 0x7FF00000u;                                   // NaN: mantissa field leading, quiet
    return sign | r;
}

// SRC / DST: bytes of one chunk before and after; UNITS: units per chunk (bytes when copying).
// A widening conversion's chunk is what one 16-byte store holds: two 16-byte stores per lane, 32
// bytes apart from lane to lane, ran at half to two thirds of the rate of one store per lane (a bare
// kernel with that access shape reaches 3.2 TB/s against 6.2 to 6.5), while two loads per lane, as
// the narrowing conversions have, cost little.
template <uint32_t CONV> struct ConvTraits {
    static constexpr uint32_t UNITS = conv_chunk_elems(CONV);
    static constexpr uint32_t SRC = UNITS * conv_src_bytes(CONV), DST = UNITS * conv_dst_bytes(CONV);
    static_assert(SRC == 4 || SRC == 8 || SRC == 16 || SRC == 32, "chunk loads come in these sizes");
    static_assert(DST == 8 || DST == 16, "one store per lane");
};
template <uint32_t CONV> constexpr bool from_e5m2 = CONV == CONV_E5H || CONV == CONV_E5B || CONV == CONV_E5F;
template <uint32_t CONV> constexpr bool from_e4m3 = CONV == CONV_E4H || CONV == CONV_E4B || CONV == CONV_E4F;

template <uint32_t CONV>
__device__ __forceinline__ uint32_t convert_bits(uint32_t v)
{
    if (CONV == CONV_H2B) return float_to_bfloat(half_to_float(v));     // one rounding: widening is exact
    if (CONV == CONV_B2H) return float_to_half(bfloat_to_float(v));
    if (CONV == CONV_H2F) return half_to_float(v);
    if (CONV == CONV_B2F) return bfloat_to_float(v);
    if (CONV == CONV_F2H) return float_to_half(v);
    if (CONV == CONV_F2B) return float_to_bfloat(v);
    if (CONV == CONV_E5H) return e5m2_to_half(v);                       // every 8-bit value is exact in all three targets
    if (CONV == CONV_E5F) return half_to_float(e5m2_to_half(v));
    if (CONV == CONV_E5B) return float_to_bfloat(half_to_float(e5m2_to_half(v)));
    if (CONV == CONV_E4F) return e4m3_to_float(v);
    if (CONV == CONV_E4H) return float_to_half(e4m3_to_float(v));
    if (CONV == CONV_E4B) return float_to_bfloat(e4m3_to_float(v));
    return v;
}

// One element of any width (the element path).
template <uint32_t CONV>
__device__ __forceinline__ uint64_t convert_element(uint64_t v)
{
    if (CONV == CONV_D2F) return double_to_float(v);
    if (CONV == CONV_F2D) return float_to_double(uint32_t(v));
    if (CONV == CONV_D2H) return float_to_half(double_to_float_odd(v));
    if (CONV == CONV_D2B) return float_to_bfloat(double_to_float_odd(v));
    if (CONV == CONV_H2D) return float_to_double(half_to_float(uint32_t(v)));
    if (CONV == CONV_B2D) return float_to_double(bfloat_to_float(uint32_t(v)));
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

// Four E5M2 bytes as two pairs of binary16 (the byte becomes the upper byte of the half).
__device__ __forceinline__ void e5m2_word_to_half_pairs(uint32_t w, uint32_t &p01, uint32_t &p23)
{
    p01 = ((w & 0x000000FFu) << 8) | ((w & 0x0000FF00u) << 16);
    p23 = ((w >> 8) & 0x0000FF00u) | (w & 0xFF000000u);
}
// Byte K of four E4M3 bytes (not the NaN) as binary32: the 7 magnitude bits placed over a binary32's
// low exponent and leading mantissa bits stand for the value times 2^-120, subnormals included
// (they land on binary32 subnormals), and the multiplication is exact.
template <uint32_t K>
__device__ __forceinline__ uint32_t e4m3_byte_to_float(uint32_t w)
{
    constexpr uint32_t UP = K == 3 ? 0u : 20u - 8u * K;                 // byte 3 moves down by 4 instead
    const uint32_t field = (K == 3 ? w >> 4 : w << UP) & 0x07F00000u;
    const uint32_t sign = (w << (24u - 8u * K)) & 0x80000000u;
    return __float_as_uint(__uint_as_float(field) * 0x1p120f) | sign;
}
// Two binary32 whose low 16 bits are zero -> two bfloat16.
__device__ __forceinline__ uint32_t upper_halves(uint32_t a, uint32_t b)
{
    return (a >> 16) | (b & 0xFFFF0000u);
}

// Four finite 8-bit floats in a word -> four binary32.
template <uint32_t CONV>
__device__ __forceinline__ u32x4 fp8_word_to_floats(uint32_t w)
{
    u32x4 r;
    if (from_e5m2<CONV>) {
        uint32_t p01, p23;
        e5m2_word_to_half_pairs(w, p01, p23);
        const f32x2 a = widen_half_pair(p01), b = widen_half_pair(p23);
        r.x = __float_as_uint(a.x); r.y = __float_as_uint(a.y); r.z = __float_as_uint(b.x); r.w = __float_as_uint(b.y);
    } else {
        r.x = e4m3_byte_to_float<0>(w); r.y = e4m3_byte_to_float<1>(w);
        r.z = e4m3_byte_to_float<2>(w); r.w = e4m3_byte_to_float<3>(w);
    }
    return r;
}
// Four finite 8-bit floats in a word -> four binary16 or bfloat16 in two words.
template <uint32_t CONV>
__device__ __forceinline__ u32x2 fp8_word_to_16bit(uint32_t w)
{
    u32x2 r;
    if (CONV == CONV_E5H) {
        uint32_t p01, p23;
        e5m2_word_to_half_pairs(w, p01, p23);
        r.x = p01;
        r.y = p23;
        return r;
    }
    const u32x4 f = fp8_word_to_floats<CONV>(w);
    if (CONV == CONV_E5B || CONV == CONV_E4B) {
        r.x = upper_halves(f.x, f.y);
        r.y = upper_halves(f.z, f.w);
    } else {
        r.x = narrow_to_half_pair(float_pair(f.x, f.y));
        r.y = narrow_to_half_pair(float_pair(f.z, f.w));
    }
    return r;
}

// True when some element of the chunk has an all-ones exponent field.  Adding the field's lowest
// bit to the masked field carries into the bit above it exactly when the field is all ones; for
// two 16-bit elements in a word the lower carry stops at bit 15, below the upper element.
template <uint32_t CONV>
__device__ __forceinline__ bool chunk_has_inf_or_nan(const Chunk32 &in)
{
    if (CONV == CONV_D2F || CONV == CONV_D2H || CONV == CONV_D2B) {
        // the exponent of a binary64 element sits in its upper word
        constexpr uint32_t MASK = 0x7FF00000u, LOW = 0x00100000u;
        const uint32_t acc = ((in.lo.y & MASK) + LOW) | ((in.lo.w & MASK) + LOW) | ((in.hi.y & MASK) + LOW) |
                             ((in.hi.w & MASK) + LOW);
        return (acc & 0x80000000u) != 0;
    }
    if (from_e5m2<CONV> || from_e4m3<CONV>) {
        // eight bytes in two words (four in one, the other word zero, for binary32 results); E5M2: exponent field all ones; E4M3: the one NaN pattern (its
        // last binade is ordinary).  The carry of a byte stops at the byte's own top bit.
        constexpr uint32_t M8 = from_e5m2<CONV> ? 0x7C7C7C7Cu : 0x7F7F7F7Fu;
        constexpr uint32_t L8 = from_e5m2<CONV> ? 0x04040404u : 0x01010101u;
        return ((((in.lo.x & M8) + L8) | ((in.lo.y & M8) + L8)) & 0x80808080u) != 0;
    }
    constexpr bool WIDE = CONV == CONV_F2H || CONV == CONV_F2B || CONV == CONV_F2D;
    constexpr bool BF = CONV == CONV_B2H || CONV == CONV_B2D;           // (bfloat16 -> binary32 never gets here)
    constexpr uint32_t MASK = WIDE ? 0x7F800000u : BF ? 0x7F807F80u : 0x7C007C00u;
    constexpr uint32_t LOW = WIDE ? 0x00800000u : BF ? 0x00800080u : 0x04000400u;
    if (ConvTraits<CONV>::SRC <= 8)                                      // up to four 16-bit or two 32-bit elements in two words (unused ones zero)
        return ((((in.lo.x & MASK) + LOW) | ((in.lo.y & MASK) + LOW)) & 0x80008000u) != 0;
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
        o.lo.x = __float_as_uint(a.x); o.lo.y = __float_as_uint(a.y);
        o.lo.z = __float_as_uint(b.x); o.lo.w = __float_as_uint(b.y);
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
        o.lo.x = uint32_t(a); o.lo.y = uint32_t(a >> 32); o.lo.z = uint32_t(b); o.lo.w = uint32_t(b >> 32);
    } else if (CONV == CONV_D2H || CONV == CONV_D2B) {
        const uint32_t a = double_to_float_odd(in.lo.x | (uint64_t(in.lo.y) << 32));
        const uint32_t b = double_to_float_odd(in.lo.z | (uint64_t(in.lo.w) << 32));
        const uint32_t c = double_to_float_odd(in.hi.x | (uint64_t(in.hi.y) << 32));
        const uint32_t d = double_to_float_odd(in.hi.z | (uint64_t(in.hi.w) << 32));
        if (CONV == CONV_D2H) {
            o.lo.x = narrow_to_half_pair(float_pair(a, b));
            o.lo.y = narrow_to_half_pair(float_pair(c, d));
        } else {
            o.lo.x = narrow_to_bfloat_pair(float_pair(a, b));
            o.lo.y = narrow_to_bfloat_pair(float_pair(c, d));
        }
    } else if (CONV == CONV_H2D || CONV == CONV_B2D) {
        const f32x2 p = CONV == CONV_H2D ? widen_half_pair(in.lo.x) : widen_bfloat_pair(in.lo.x);
        const uint64_t a = uint64_t(__double_as_longlong(double(p.x))), b = uint64_t(__double_as_longlong(double(p.y)));
        o.lo.x = uint32_t(a); o.lo.y = uint32_t(a >> 32); o.lo.z = uint32_t(b); o.lo.w = uint32_t(b >> 32);
    } else if (CONV == CONV_E5F || CONV == CONV_E4F) {
        o.lo = fp8_word_to_floats<CONV>(in.lo.x);                       // four bytes in a word -> four binary32
    } else if (from_e5m2<CONV> || from_e4m3<CONV>) {
        // eight bytes in two words -> eight 16-bit elements
        const u32x2 a = fp8_word_to_16bit<CONV>(in.lo.x), b = fp8_word_to_16bit<CONV>(in.lo.y);
        o.lo.x = a.x; o.lo.y = a.y; o.lo.z = b.x; o.lo.w = b.y;
    }
    return o;
}

// The four 8-bit floats of a word converted one by one, whatever they hold.
template <uint32_t CONV>
__device__ __forceinline__ u32x4 fp8_word_any(uint32_t w)
{
    u32x4 r;
    r.x = convert_bits<CONV>(w & 0xFFu);
    r.y = convert_bits<CONV>((w >> 8) & 0xFFu);
    r.z = convert_bits<CONV>((w >> 16) & 0xFFu);
    r.w = convert_bits<CONV>(w >> 24);
    return r;
}

// One chunk (2 to 8 elements, or 16 raw bytes) in, converted out.
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
    } else if (CONV == CONV_D2F) {
        o.lo.x = double_to_float(in.lo.x | (uint64_t(in.lo.y) << 32));
        o.lo.y = double_to_float(in.lo.z | (uint64_t(in.lo.w) << 32));
        o.lo.z = double_to_float(in.hi.x | (uint64_t(in.hi.y) << 32));
        o.lo.w = double_to_float(in.hi.z | (uint64_t(in.hi.w) << 32));
    } else if (CONV == CONV_F2D) {
        const uint64_t a = float_to_double(in.lo.x), b = float_to_double(in.lo.y);
        o.lo.x = uint32_t(a); o.lo.y = uint32_t(a >> 32); o.lo.z = uint32_t(b); o.lo.w = uint32_t(b >> 32);
    } else if (CONV == CONV_D2H || CONV == CONV_D2B) {
        const uint32_t a = uint32_t(convert_element<CONV>(in.lo.x | (uint64_t(in.lo.y) << 32)));
        const uint32_t b = uint32_t(convert_element<CONV>(in.lo.z | (uint64_t(in.lo.w) << 32)));
        const uint32_t c = uint32_t(convert_element<CONV>(in.hi.x | (uint64_t(in.hi.y) << 32)));
        const uint32_t d = uint32_t(convert_element<CONV>(in.hi.z | (uint64_t(in.hi.w) << 32)));
        o.lo.x = a | (b << 16);
        o.lo.y = c | (d << 16);
    } else if (CONV == CONV_H2D || CONV == CONV_B2D) {
        const uint64_t a = convert_element<CONV>(in.lo.x & 0xFFFFu), b = convert_element<CONV>(in.lo.x >> 16);
        o.lo.x = uint32_t(a); o.lo.y = uint32_t(a >> 32); o.lo.z = uint32_t(b); o.lo.w = uint32_t(b >> 32);
    } else if (CONV == CONV_E5F || CONV == CONV_E4F) {
        o.lo = fp8_word_any<CONV>(in.lo.x);
    } else if (from_e5m2<CONV> || from_e4m3<CONV>) {
        const u32x4 a = fp8_word_any<CONV>(in.lo.x), b = fp8_word_any<CONV>(in.lo.y);
        o.lo.x = a.x | (a.y << 16); o.lo.y = a.z | (a.w << 16); o.lo.z = b.x | (b.y << 16); o.lo.w = b.z | (b.w << 16);
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
    __device__ __forceinline__ uint32_t unit0() const { return w[13]; }
    __device__ __forceinline__ uint32_t grain() const { return w[14]; }
    __device__ __forceinline__ uint32_t staged() const { return w[15]; }
};
static_assert(offsetof(DevDesc, src_off) == 0 && offsetof(DevDesc, src_stride) == 8 && offsetof(DevDesc, dst) == 16 &&
              offsetof(DevDesc, n_units) == 24 && offsetof(DevDesc, units_per_row) == 32 &&
              offsetof(DevDesc, tile0) == 36 && offsetof(DevDesc, n_tiles) == 40 && offsetof(DevDesc, div_m) == 44 &&
              offsetof(DevDesc, div_s) == 48 && offsetof(DevDesc, unit0) == 52 && offsetof(DevDesc, grain) == 56 &&
              offsetof(DevDesc, staged) == 60,
              "PieceRegs reads DevDesc by dword position");

// The piece that owns tile `b`.  hints[k] names the piece that holds the first tile of span k (a span
// is 2^shift tiles; past the end: the last piece), so the owner lies between hints[b >> shift] and
// the next entry: for a span inside one tensor the two are equal and nothing is searched; a span
// that holds several small tensors costs a binary search over first-tile fields (the host picks the
// span so that it holds two pieces at most on average).
__device__ __forceinline__ PieceRegs find_piece(const DevDesc *__restrict__ descs,
                                                const uint32_t *__restrict__ hints, uint32_t b, uint32_t shift)
{
    uint32_t lo = hints[b >> shift], hi = hints[(b >> shift) + 1];
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

// What a wavefront works on: its tile's piece, the tile's first chunk inside the piece and the
// number of chunks the tile holds (64 but for a piece's last tile).  Workgroup position p of the
// launch (see tile_of_workgroup) takes tiles p*WG_TILES .. p*WG_TILES+15, one per wavefront; all
// of it depends on the workgroup and wavefront index alone, so it lives in scalar registers.
struct WaveTile {
    PieceRegs d;
    uint32_t c0, n;
};
__device__ __forceinline__ bool wave_tile(const DevDesc *__restrict__ descs, const uint32_t *__restrict__ hints,
                                          uint32_t wg_base, uint32_t hint_shift, WaveTile &wt)
{
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const uint32_t b = (wg_base + tile_of_workgroup(blockIdx.x, gridDim.x)) * WG_TILES + wave;
    // The launch's last workgroup may reach past the launch's last tile.  The hint table covers those
    // tile indices too and leads them to the last piece, where they show as tiles past its end:
    // telling them apart here, before the lookup, would put one more dependent scalar load (the
    // tile count) in front of the wavefront's first memory access.
    wt.d = find_piece(descs, hints, b, hint_shift);
    const uint32_t t = b - wt.d.tile0();                                // tile inside the piece
    if (t >= wt.d.n_tiles()) return false;
    wt.c0 = t * VEC_TILE_UNITS;                                         // a piece has at most 2^31 chunks
    // only a piece's last tile can be short; decided on 32-bit tile counts
    wt.n = (t + 1 == wt.d.n_tiles()) ? uint32_t(wt.d.n_units()) - wt.c0 : VEC_TILE_UNITS;
    return true;
}

template <uint32_t CS, bool BYTE, bool FUSED>
__device__ __forceinline__ Chunk32 load_chunk(const uint8_t *s)
{
    Chunk32 v;
    if (CS == 4) v.lo = load4<BYTE, FUSED>(s);
    else if (CS == 8) v.lo = load8<BYTE, FUSED>(s);
    else if (CS == 16) v.lo = load16<BYTE>(s);
    else v = load32<BYTE>(s);
    return v;
}

template <uint32_t CD>
__device__ __forceinline__ void store_chunk(uint8_t *t, const Chunk32 &o)
{
    static_assert(CD == 8 || CD == 16, "one store per lane");
    if (CD == 8) gstore8(t, o.lo.x, o.lo.y);
    else gstore16(t, o.lo);
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
    const Chunk32 o = convert_chunk<CONV>(load_chunk<CS, BYTE, true>(s));
    store_chunk<CD>(dst + uint64_t(c) * CD, o);
}

template <uint32_t CONV, bool BYTE>
__global__ __launch_bounds__(VEC_BLOCK_THREADS) void materialize_vec(const DevDesc *__restrict__ descs,
                                                                     const uint32_t *__restrict__ hints,
                                                                     const uint8_t *__restrict__ raw,
                                                                     uint32_t wg_base, uint32_t hint_shift)
{
    WaveTile wt;
    if (!wave_tile(descs, hints, wg_base, hint_shift, wt)) return;
    const uint32_t lane = threadIdx.x % WAVE;
    if (lane < wt.n)
        vec_chunk<CONV, BYTE>(raw + wt.d.src_off(), reinterpret_cast<uint8_t *>(wt.d.dst()), wt.c0 + lane, wt.d);
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
// say, 2050 bytes).  The output is one contiguous stream; a lane owns one aligned chunk of it,
// i.e. CH consecutive units (bytes when copying, elements when converting); the piece's first unit
// is unit unit0 of its first row (a piece starts on a store boundary of the output, which need not
// be the start of a row).  Most chunks lie inside one row and are read like a byte-aligned vector
// chunk.  A chunk that straddles a row end takes its first k units from the end of row r and the
// rest from the start of row r+1: the second read starts k units *before* row r+1 (inside row r's
// stride, since a row has at least CH units), so that both reads hold their units at the chunk's
// own positions and a byte mask splices them.
template <uint32_t CONV>
__global__ __launch_bounds__(VEC_BLOCK_THREADS) void materialize_splice(const DevDesc *__restrict__ descs,
                                                                        const uint32_t *__restrict__ hints,
                                                                        const uint8_t *__restrict__ raw,
                                                                        uint32_t wg_base, uint32_t hint_shift)
{
    constexpr uint32_t CS = ConvTraits<CONV>::SRC, CD = ConvTraits<CONV>::DST;
    constexpr uint32_t CH = ConvTraits<CONV>::UNITS;                    // units per chunk
    constexpr uint32_t US = CS / CH;                                    // source bytes per unit
    WaveTile wt;
    if (!wave_tile(descs, hints, wg_base, hint_shift, wt)) return;
    const PieceRegs &d = wt.d;
    const uint32_t lane = threadIdx.x % WAVE;
    if (lane >= wt.n) return;
    const uint32_t c = wt.c0 + lane;
    const uint32_t u0 = d.unit0() + c * CH;                             // the piece ends below unit 2^31
    const uint32_t upr = d.units_per_row();
    const uint32_t r = fast_div(u0, d.div_m(), d.div_s());
    const uint32_t col = u0 - r * upr;
    const uint8_t *row = raw + d.src_off() + uint64_t(r) * d.src_stride();
    Chunk32 v = load_chunk<CS, true, false>(row + uint64_t(col) * US);
    const uint32_t k = upr - col;                                       // units left in row r
    if (k < CH) {
        const uint8_t *next = row + d.src_stride() - k * US;
        const Chunk32 w = load_chunk<CS, true, false>(next);
        v = splice_chunk<CS>(v, w, k * US);
    }
    const Chunk32 o = convert_chunk<CONV>(v);
    store_chunk<CD>(reinterpret_cast<uint8_t *>(d.dst()) + uint64_t(c) * CD, o);
}

// One unit of G bytes (1, 2, 4 or 8) from an address that is a multiple of G.
template <uint32_t G>
__device__ __forceinline__ uint64_t load_unit(const uint8_t *p)
{
    if (G == 1) return *(const FST_GLOBAL uint8_t *)(p);
    if (G == 2) return *(const FST_GLOBAL uint16_t *)(p);
    if (G == 4) return *(const FST_GLOBAL uint32_t *)(p);
    return *(const FST_GLOBAL uint64_t *)(p);
}
// One element of ES bytes from any address, byte by byte.
template <uint32_t ES>
__device__ __forceinline__ uint64_t load_bytes(const uint8_t *p)
{
    uint64_t v = 0;
#pragma unroll
    for (uint32_t k = 0; k < ES; ++k) v |= uint64_t(*(const FST_GLOBAL uint8_t *)(p + k)) << (8 * k);
    return v;
}
// OR v into 32-bit word `word` of a chunk seen as eight words.
__device__ __forceinline__ void chunk_or(Chunk32 &c, uint32_t word, uint32_t v)
{
    switch (word) {                                     // `word` is a compile-time constant after unrolling
    case 0: c.lo.x |= v; break;
    case 1: c.lo.y |= v; break;
    case 2: c.lo.z |= v; break;
    case 3: c.lo.w |= v; break;
    case 4: c.hi.x |= v; break;
    case 5: c.hi.y |= v; break;
    case 6: c.hi.z |= v; break;
    default: c.hi.w |= v; break;
    }
}

// G consecutive source bytes of one row, starting at byte u of the piece's byte stream (copying).
template <uint32_t G>
__device__ __forceinline__ uint64_t gather_bytes(const uint8_t *base, const PieceRegs &d, uint32_t u)
{
    const uint32_t r = fast_div(u, d.div_m(), d.div_s());
    return load_unit<G>(base + uint64_t(r) * d.src_stride() + (u - r * d.units_per_row()));
}

// Gather path: rows shorter than one chunk (a partition along the last dimension of a tensor whose
// rows are a few elements long).  As in the spliced path a lane owns one aligned chunk of the
// output stream, but its units come from several rows, so it fetches them one by one: with loads
// of `grain` bytes when the geometry keeps every source address a multiple of it (1, 2, 4 or 8
// bytes; one element at a time when converting), byte by byte otherwise.  The stores are
// full-width.  Neighbouring lanes read neighbouring rows, so every cache line is still fetched
// once; what bounds this path is that a line is fetched whole for the few bytes kept of it.
// Loads of 4 bytes and less are many scattered addresses per wavefront, which the address units
// take a few per cycle: where a tile's whole source span fits (shares of a half to a quarter of a
// row, roughly), the wavefront reads the span with coalesced 16-byte loads into LDS instead and
// the lanes pick their bytes out of it (2.9 to 3.1 TB/s against 1.4 to 2.2).
template <uint32_t CONV>
__global__ __launch_bounds__(VEC_BLOCK_THREADS) void materialize_gather(const DevDesc *__restrict__ descs,
                                                                        const uint32_t *__restrict__ hints,
                                                                        const uint8_t *__restrict__ raw,
                                                                        uint32_t wg_base, uint32_t hint_shift)
{
    constexpr uint32_t CS = ConvTraits<CONV>::SRC, CD = ConvTraits<CONV>::DST;
    constexpr uint32_t CH = ConvTraits<CONV>::UNITS;
    constexpr uint32_t US = CS / CH;
    __shared__ __attribute__((aligned(16))) uint8_t lds[WG_TILES * GATHER_LDS_BYTES];
    WaveTile wt;
    if (!wave_tile(descs, hints, wg_base, hint_shift, wt)) return;
    const PieceRegs &d = wt.d;
    const uint32_t lane = threadIdx.x % WAVE;
    const uint32_t c = wt.c0 + lane;
    const uint32_t u0 = d.unit0() + c * CH;
    const uint8_t *base = raw + d.src_off();
    const uint32_t grain = d.grain();
    Chunk32 v;
    v.lo = u32x4{0u, 0u, 0u, 0u};
    v.hi = u32x4{0u, 0u, 0u, 0u};
    if (d.staged()) {
        // The tile's units [t0, t1] lie in rows r0 .. r1.  Everything from the first wanted byte
        // (rounded down to a dword) to the last (rounded up) is read once, coalesced, into this
        // wavefront's LDS area: the host has checked that it fits for every tile of the piece.
        const uint32_t upr = d.units_per_row(), stride = uint32_t(d.src_stride());
        const uint32_t t0 = d.unit0() + wt.c0 * CH, t1 = t0 + wt.n * CH - 1;
        const uint32_t r0 = fast_div(t0, d.div_m(), d.div_s()), r1 = fast_div(t1, d.div_m(), d.div_s());
        const uint32_t col0 = t0 - r0 * upr, col1 = t1 - r1 * upr;
        const uintptr_t first = reinterpret_cast<uintptr_t>(base) + uint64_t(r0) * stride + col0 * US;
        const uint8_t *from = reinterpret_cast<const uint8_t *>(first & ~uintptr_t(3));
        const uint32_t lead = uint32_t(first) & 3u;
        const uint32_t span = (lead + (r1 - r0) * stride + (col1 + 1 - col0) * US + 3u) & ~3u;
        uint8_t *mine = lds + __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE) * GATHER_LDS_BYTES;
        if (span <= GATHER_LDS_BYTES) {
#pragma unroll
            for (uint32_t k = 0; k < GATHER_LDS_BYTES / (16 * WAVE); ++k) {
                const uint32_t off = 16 * (lane + WAVE * k);
                if (off + 16 <= span) {
                    *reinterpret_cast<u32x4 *>(mine + off) = gload16(from + off);
                } else {
                    for (uint32_t w = off; w < span && w < off + 16; w += 4)      // the span's last, partial 16 bytes
                        *reinterpret_cast<uint32_t *>(mine + w) = gload4(from + w);
                }
            }
            // the wavefront's own writes, read back by other lanes of the same wavefront
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            if (lane >= wt.n) return;
            // byte of unit (r, col) in the area: lead + (r - r0) * stride + (col - col0) * US, never negative
            // (a unit of row r0 has col >= col0); found by division for the chunk's first unit, then stepped
            const uint32_t r = fast_div(u0, d.div_m(), d.div_s());
            uint32_t col = u0 - r * upr;
            uint32_t at = lead + (r - r0) * stride + col * US - col0 * US;
            const uint32_t to_next_row = stride - upr * US;
#pragma unroll
            for (uint32_t j = 0; j < CH; ++j) {
                uint64_t e = 0;
#pragma unroll
                for (uint32_t k = 0; k < US; ++k) e |= uint64_t(mine[at + k]) << (8 * k);
                if (US == 1) chunk_or(v, j / 4, uint32_t(e) << (8 * (j % 4)));
                else if (US == 2) chunk_or(v, j / 2, uint32_t(e) << (16 * (j % 2)));
                else if (US == 4) chunk_or(v, j, uint32_t(e));
                else { chunk_or(v, 2 * j, uint32_t(e)); chunk_or(v, 2 * j + 1, uint32_t(e >> 32)); }
                at += US;
                if (++col == upr) { col = 0; at += to_next_row; }
            }
            const Chunk32 o = convert_chunk<CONV>(v);
            store_chunk<CD>(reinterpret_cast<uint8_t *>(d.dst()) + uint64_t(c) * CD, o);
            return;
        }
    }
    if (lane >= wt.n) return;
    if (CONV == CONV_COPY) {
        // 16 bytes; rows, strides and the first address are multiples of `grain`, so `grain`
        // consecutive bytes never leave their row
        if (grain >= 8) {
#pragma unroll
            for (uint32_t j = 0; j < 2; ++j) {
                const uint64_t e = gather_bytes<8>(base, d, u0 + 8 * j);
                chunk_or(v, 2 * j, uint32_t(e));
                chunk_or(v, 2 * j + 1, uint32_t(e >> 32));
            }
        } else if (grain == 4) {
#pragma unroll
            for (uint32_t j = 0; j < 4; ++j) chunk_or(v, j, uint32_t(gather_bytes<4>(base, d, u0 + 4 * j)));
        } else if (grain == 2) {
#pragma unroll
            for (uint32_t j = 0; j < 8; ++j) chunk_or(v, j / 2, uint32_t(gather_bytes<2>(base, d, u0 + 2 * j)) << (16 * (j % 2)));
        } else {
#pragma unroll
            for (uint32_t j = 0; j < 16; ++j) chunk_or(v, j / 4, uint32_t(gather_bytes<1>(base, d, u0 + j)) << (8 * (j % 4)));
        }
    } else {
        const bool aligned = grain >= US;
#pragma unroll
        for (uint32_t j = 0; j < CH; ++j) {
            const uint32_t u = u0 + j;
            const uint32_t r = fast_div(u, d.div_m(), d.div_s());
            const uint8_t *p = base + uint64_t(r) * d.src_stride() + uint64_t(u - r * d.units_per_row()) * US;
            const uint64_t e = aligned ? load_unit<US>(p) : load_bytes<US>(p);
            if (US == 1) chunk_or(v, j / 4, uint32_t(e) << (8 * (j % 4)));
            else if (US == 2) chunk_or(v, j / 2, uint32_t(e) << (16 * (j % 2)));
            else if (US == 4) chunk_or(v, j, uint32_t(e));
            else { chunk_or(v, 2 * j, uint32_t(e)); chunk_or(v, 2 * j + 1, uint32_t(e >> 32)); }
        }
    }
    const Chunk32 o = convert_chunk<CONV>(v);
    store_chunk<CD>(reinterpret_cast<uint8_t *>(d.dst()) + uint64_t(c) * CD, o);
}

// Element path: the few units in front of a piece's first store boundary and behind its last whole
// chunk, and rows too long for the 32-bit unit indices of the other paths.  One element (one byte
// when nothing is converted) per thread and step; sources are read bytewise; indices are 64-bit.
template <uint32_t CONV>
__global__ __launch_bounds__(ELEM_BLOCK_THREADS) void materialize_elem(const DevDesc *__restrict__ descs,
                                                                       const uint32_t *__restrict__ hints,
                                                                       const uint8_t *__restrict__ raw,
                                                                       uint32_t wg_base, uint32_t hint_shift)
{
    constexpr uint32_t ES = ConvTraits<CONV>::SRC / ConvTraits<CONV>::UNITS;         // bytes per source element
    constexpr uint32_t ED = ConvTraits<CONV>::DST / ConvTraits<CONV>::UNITS;
    const uint32_t b = wg_base + blockIdx.x;                                         // one tile per workgroup
    const PieceRegs d = find_piece(descs, hints, b, hint_shift);
    const uint32_t t = b - d.tile0();
    const uint64_t e0 = uint64_t(t) * ELEM_TILE_UNITS;
    const uint32_t n = (t + 1 == d.n_tiles()) ? uint32_t(d.n_units() - e0) : ELEM_TILE_UNITS;
    const uint32_t upr = d.units_per_row();
    const uint64_t stride = d.src_stride();
    const uint64_t g0 = uint64_t(d.unit0()) + e0;                                    // counted from the start of the piece's first row
    const uint64_t row0 = g0 / upr;
    const uint32_t col0 = uint32_t(g0 - row0 * upr);
    const uint8_t *src = raw + d.src_off() + row0 * stride;
    uint8_t *dst = reinterpret_cast<uint8_t *>(d.dst()) + e0 * ED;
    for (uint32_t i = threadIdx.x; i < n; i += ELEM_BLOCK_THREADS) {
        const uint64_t cc = uint64_t(col0) + i;
        const uint64_t r = cc / upr;
        const uint8_t *s = src + r * stride + (cc - r * upr) * ES;
        const uint64_t v = convert_element<CONV>(load_bytes<ES>(s));
        uint8_t *o = dst + uint64_t(i) * ED;
        if (ED == 1) *(FST_GLOBAL uint8_t *)(o) = uint8_t(v);
        else if (ED == 2) *(FST_GLOBAL uint16_t *)(o) = uint16_t(v);
        else if (ED == 4) *(FST_GLOBAL uint32_t *)(o) = uint32_t(v);
        else *(FST_GLOBAL uint64_t *)(o) = v;
    }
}

template <uint32_t CONV>
int launch_conv(uint32_t path, bool byte_aligned, const DevDesc *descs, const uint32_t *hints, uint32_t n_tiles,
                uint32_t hint_shift, const uint8_t *raw, hipStream_t stream)
{
    for (const LaunchPart &part : split_launch(workgroups_of(path, n_tiles))) {
        const dim3 grid(part.n_wg);
        const uint32_t base = part.wg_base;
        if (path == PATH_VEC && !byte_aligned)
            hipLaunchKernelGGL((materialize_vec<CONV, false>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw,
                               base, hint_shift);
        else if (path == PATH_VEC)
            hipLaunchKernelGGL((materialize_vec<CONV, true>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw,
                               base, hint_shift);
        else if (path == PATH_SPLICE)
            hipLaunchKernelGGL((materialize_splice<CONV>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw,
                               base, hint_shift);
        else if (path == PATH_GATHER)
            hipLaunchKernelGGL((materialize_gather<CONV>), grid, dim3(VEC_BLOCK_THREADS), 0, stream, descs, hints, raw,
                               base, hint_shift);
        else
            hipLaunchKernelGGL((materialize_elem<CONV>), grid, dim3(ELEM_BLOCK_THREADS), 0, stream, descs, hints, raw,
                               base, hint_shift);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(FST_E_HIP, "kernel launch failed: %s", hipGetErrorString(e));
    }
    return FST_OK;
}

// launch_conv<C> for the C that equals `conv`.
template <uint32_t... C, typename... Args>
int launch_any_conv(uint32_t conv, std::integer_sequence<uint32_t, C...>, Args... args)
{
    int rc = FST_E_ARG;
    const bool found = ((conv == C ? (rc = launch_conv<C>(args...), true) : false) || ...);
    return found ? rc : fail(FST_E_ARG, "unknown conversion %u", conv);
}

}  // namespace

int launch_class_kernels(uint32_t cls, const DevDesc *descs_dev, const uint32_t *hints_dev, uint32_t n_tiles,
                         uint32_t hint_shift, const void *raw_dev, void *stream)
{
    if (n_tiles == 0) return FST_OK;
    if (cls >= N_CLASSES) return fail(FST_E_ARG, "unknown launch class %u", cls);
    const uint32_t path = class_path(cls), conv = class_conv(cls);
    const bool byte_aligned = path == PATH_VEC && cls % 2 == 1;
    const uint8_t *raw = static_cast<const uint8_t *>(raw_dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    return launch_any_conv(conv, std::make_integer_sequence<uint32_t, CONV_COUNT>{}, path, byte_aligned, descs_dev, hints_dev, n_tiles,
                           hint_shift, raw, s);
}

}  // namespace fst
