// Device code of the mxc library for gfx950 (wave64).
//
// Every kernel treats a tensor [tokens x hidden] as a flat array (blocks never straddle rows
// because hidden % block == 0, and rows are packed back to back, so the flat view of inputs,
// packed codes and scales is exact).  A "unit" is 8 consecutive elements: one 128-bit load of
// bf16, one dword of 4-bit codes, b bytes of b-bit codes.  In the quantize kernels a block of B
// elements is B/8 neighbouring lanes of one wave (1, 2 or 4 lanes), so the block maximum is a
// quad-local DPP reduction and never touches LDS; each wave owns U * 64 consecutive units and in
// step u lane l handles unit (wave_base + u*64 + l), which keeps every load and store instruction
// contiguous across the wave.  The reduce kernels give a lane a chunk of 32 consecutive elements
// (tile form) or half of one (half-chunk form); see their sections.
//
// Element rounding and decoding use the gfx950 scaled-conversion instructions wherever the
// element format maps onto a hardware format bit for bit (checked exhaustively against the CPU
// oracle): E2M1 is the hardware FP4; a format with 2 (3) mantissa bits is the low part of the
// code space of BF8 = E5M2 (FP8 = E4M3) once the block scale is shifted so that the smallest
// normals coincide; for decoding, a block of 32 E3M2 codes is one hardware BF6 block and a block
// of 32 E2M3 or (widened by one zero bit per code) E2M2 codes one hardware FP6 block.  Everything
// else, and every block whose scale leaves the range in which that shift is representable, takes
// the integer path below, which is exact for every input.
//
// This file: types, the element and scale formats, rounding and bit-stream helpers shared by the
// quantize and reduce kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

namespace mxc {

constexpr int kThreads = 256;        // 4 waves per workgroup

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x32 __attribute__((ext_vector_type(32)));
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

enum HwKind { HW_NONE = 0, HW_FP4 = 1, HW_BF8 = 2, HW_FP8 = 3 };

// Element format ExMy (Method, parameter list): facts derived at compile time.
template <int X, int Y>
struct Elem {
    static constexpr int x = X, y = Y;
    static constexpr int bits = 1 + X + Y;
    static constexpr int beta = (1 << (X - 1)) - 1;
    static constexpr int emax = (1 << X) - 1 - beta;
    static constexpr uint32_t magmask = (1u << (X + Y)) - 1u;
    // hardware format whose code space contains this one
    static constexpr int hw = (X == 2 && Y == 1) ? HW_FP4 : (Y == 2) ? HW_BF8 : (Y == 3) ? HW_FP8
                                                                                       : HW_NONE;
    // exponent bias of that hardware format
    static constexpr int hw_bias = hw == HW_BF8 ? 15 : hw == HW_FP8 ? 7 : beta;
    // Decoding only: a format with one mantissa bit is also part of BF8's code space once its
    // mantissa is padded with a zero bit (same values; not usable for rounding, which would
    // round twice).  dec_pad: zero bits to append to the magnitude.
    static constexpr int dec_pad = (hw == HW_NONE && Y == 1) ? 1 : 0;
    static constexpr int hw_dec = dec_pad ? HW_BF8 : hw;
    static constexpr int hw_dec_bias = dec_pad ? 15 : hw_bias;
};

// Scale format EsM0, runtime (s only changes two clamps per block).
struct ScaleFmt {
    int sbits;      // s: 8 = one byte per block; 4..7 = packed s-bit stream, LSB first
    int sbias;      // 2^(s-1) - 1
    int smax;       // largest ordinary code: 254 for s = 8, 2^s - 1 otherwise
    int nonfinite;  // code stored for a block that held Inf/NaN: 255 for s = 8, smax otherwise
    int has_nan;    // 1 when code 255 decodes to NaN (s = 8)
};

constexpr int quad_perm(int a, int b, int c, int d) { return a | (b << 2) | (c << 4) | (d << 6); }

template <int CTRL>
__device__ __forceinline__ uint32_t dpp(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, true);
}

__device__ __forceinline__ uint32_t pk_max_u16(uint32_t a, uint32_t b)
{
    u16x2 r = __builtin_elementwise_max(__builtin_bit_cast(u16x2, a), __builtin_bit_cast(u16x2, b));
    return __builtin_bit_cast(uint32_t, r);
}

// Two bfloat16 in a dword, as the vector type the conversion builtins take.  The argument is a
// by-value scalar on purpose: bit-casting an element of a vector variable in place made the
// compiler read element 0 for every index.
__device__ __forceinline__ bf16x2 as_bf16x2(uint32_t pair)
{
    bf16x2 r;
    __builtin_memcpy(&r, &pair, sizeof(r));
    return r;
}

template <bool NT, class T>
__device__ __forceinline__ T ld(const T *p)
{
    return NT ? __builtin_nontemporal_load(p) : *p;
}

template <bool NT, class T>
__device__ __forceinline__ void st(T *p, T v)
{
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// Maximum over the B/8 lanes that share a block.
template <int B>
__device__ __forceinline__ uint32_t block_max(uint32_t m)
{
    if (B >= 16) m = max(m, dpp<quad_perm(1, 0, 3, 2)>(m));
    if (B >= 32) m = max(m, dpp<quad_perm(2, 3, 0, 1)>(m));
    return m;
}

// ---------------------------------------------------------------------------------------------
// Integer-path rounding of one element to an ExMy magnitude code, ties to the even code,
// saturating.
//
// round_small_sig: for inputs with at most 8 significant bits (bfloat16).  The value is scaled
// by 2^(beta-127-e) so that the element format's smallest normal lands on binary32's smallest
// normal; the binary32 bit pattern of the result is then the element code followed by 23-y
// extra fraction bits, continuously across the subnormal/normal boundary, and a single integer
// round-half-even of those extra bits finishes the job.  The scaling is exact: a result with
// fewer than 8 bits of room above 2^-149 is below 2^-141, far under half the smallest step.
template <class E>
__device__ __forceinline__ uint32_t round_small_sig(float v, int k /* beta - 127 - e */)
{
    uint32_t u = __float_as_uint(ldexpf(__builtin_fabsf(v), k));
    constexpr int sh = 23 - E::y;
    uint32_t r = (u + ((1u << (sh - 1)) - 1u) + ((u >> sh) & 1u)) >> sh;
    return min(r, E::magmask);
}

// round_full_sig: for binary32 inputs (24 significant bits), where the scaling above could lose
// sticky bits.  p = |v| * 2^-e is exact in the normal range; a magnitude that is normal in the
// element format is rounded on its bit pattern, a subnormal one by one binary32 add of
// 2^(1-beta-y+23), whose unit in the last place is the subnormal step.
template <class E>
__device__ __forceinline__ uint32_t round_full_sig(float v, int neg_e)
{
    float p = ldexpf(__builtin_fabsf(v), neg_e);
    constexpr int sh = 23 - E::y;
    uint32_t u = __float_as_uint(p);
    uint32_t rn = ((u + ((1u << (sh - 1)) - 1u) + ((u >> sh) & 1u)) >> sh) -
                  ((uint32_t)(127 - E::beta) << E::y);
    const float magic = __uint_as_float((uint32_t)(1 - E::beta - E::y + 23 + 127) << 23);
    uint32_t rs = __float_as_uint(p + magic) - __float_as_uint(magic);
    const float min_normal = __uint_as_float((uint32_t)(1 - E::beta + 127) << 23);
    uint32_t r = p < min_normal ? rs : rn;
    return min(r, E::magmask);
}

// ---------------------------------------------------------------------------------------------
// Four bytes of a dword (code k in byte k, each below 2^b) -> four b-bit fields.
template <int BITS>
__device__ __forceinline__ uint32_t squeeze4(uint32_t bytes)
{
    constexpr uint32_t m1 = (1u << BITS) - 1u, m2 = (1u << 2 * BITS) - 1u;
    // bytes 0,1 -> 2b bits in the low half, bytes 2,3 -> 2b bits in the high half
    uint32_t t = (bytes & (m1 * 0x00010001u)) | ((bytes >> (8 - BITS)) & ((m1 << BITS) * 0x00010001u));
    return (t & m2) | ((t >> (16 - 2 * BITS)) & (m2 << 2 * BITS));
}

// ---------------------------------------------------------------------------------------------
// Moving b-bit codes between "8 codes per lane" and the packed little-endian bit stream.
// A quad of lanes owns 32 codes = b dwords of the stream, at dword index quad*b.

// How many bytes of the quad's b dwords lie inside the array: the last quad of a tensor whose
// size is not a multiple of 32 elements holds fewer than four units.
__device__ __forceinline__ int quad_valid_bytes(size_t unit, size_t units_total, int bits)
{
    const size_t q0 = unit & ~(size_t)3;
    const size_t left = units_total > q0 ? units_total - q0 : 0;
    return (int)(left < 4 ? left : 4) * bits;
}

// Stores the first `nbytes` bytes of dword v at p (all four when nbytes >= 4, none when <= 0).
template <bool NT>
__device__ __forceinline__ void store_prefix(uint32_t *p, uint32_t v, int nbytes)
{
    if (nbytes >= 4) {
        // the same kind of store as the full-quad path: the compiler merges the two, and a merge
        // of a nontemporal store with a plain one would come out plain
        st<NT>(p, v);
    } else {
        for (int k = 0; k < nbytes; ++k) ((uint8_t *)p)[k] = (uint8_t)(v >> (8 * k));
    }
}

// Store: lane holds its 8 codes in the low 8b bits of v (zero for a unit past the end).  After
// the in-quad exchange each lane owns up to two whole dwords of the stream (k0, k1; -1 = none).
template <int BITS, bool NT>
__device__ __forceinline__ void store_codes(uint32_t *codes, size_t unit, uint64_t v, size_t units_total)
{
    const int i = (int)(threadIdx.x & 3);
    if (BITS == 4) {
        if (unit < units_total) st<NT>(codes + unit, (uint32_t)v);
        return;
    }
    int k0 = -1, k1 = -1;
    uint32_t d0 = 0, d1 = 0;
    if (BITS == 5) {
        // lane i's 40 bits start at stream bit 40i = dword i, bit 8i
        uint64_t w = v << (8 * i);
        uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
        uint32_t from_prev = dpp<quad_perm(3, 0, 1, 2)>(hi);     // lane i gets hi of lane i-1
        k0 = i;
        d0 = lo | (i ? from_prev : 0u);
        if (i == 0) {                                            // hi of lane 3
            k1 = 4;
            d1 = from_prev;
        }
    } else if (BITS == 6) {
        // pairs of lanes own 3 dwords: even lane bits 0..47, odd lane bits 48..95
        uint64_t w = v << (16 * (i & 1));
        uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
        uint32_t give = (i & 1) ? lo : hi;
        uint32_t got = dpp<quad_perm(1, 0, 3, 2)>(give);          // odd lane gets even's hi
        const int p0 = 3 * (i >> 1);                              // first dword of the pair
        if (i & 1) {
            k0 = p0 + 1;
            d0 = lo | got;
            k1 = p0 + 2;
            d1 = hi;
        } else {
            k0 = p0;
            d0 = lo;
        }
    } else {  // BITS == 3: lane i's 24 bits start at stream bit 24i
        const int s = (32 - 8 * i) & 31;                          // 0, 24, 16, 8
        uint64_t w = v << s;
        uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
        uint32_t from_next = dpp<quad_perm(1, 2, 3, 3)>(lo);      // lane i gets lo of lane i+1
        if (i < 3) {
            k0 = i;
            d0 = (i ? hi : lo) | from_next;
        }
    }
    uint32_t *q = codes + (unit >> 2) * BITS;
    if ((unit | 3) < units_total) {                               // the whole quad is inside
        if (k0 >= 0) st<NT>(q + k0, d0);
        if (k1 >= 0) st<NT>(q + k1, d1);
    } else {                                                      // the tensor's last, partial quad
        const int vb = quad_valid_bytes(unit, units_total, BITS);
        if (k0 >= 0) store_prefix<NT>(q + k0, d0, vb - 4 * k0);
        if (k1 >= 0) store_prefix<NT>(q + k1, d1, vb - 4 * k1);
    }
}

// ---------------------------------------------------------------------------------------------
// Narrow scale formats (s < 8) travel as a bit stream: block k's code at bits [k*s, (k+1)*s) of
// the tensor's scale array, LSB first, the last byte padded with zeros.

// Wave-wide store of 64/G consecutive fields of WIDTH bits (4..28), field f held by lane f*G in
// `value` (fields past `nvalid` must hold 0).  `dst` is the byte where field 0 starts, which is
// always a byte boundary because 64/G fields of any width fill a whole number of bytes.  Lane j
// assembles byte j (and j+64, ... for wide fields) from the up to three fields that overlap it.
// Every lane of the wave must call this, and every lane runs the same number of rounds: the
// cross-lane reads need their source lanes active.
// WIDTH is a compile-time constant so that the division below folds into a multiply (with a
// run-time width it costs some 40 instructions per call).
template <int G, int WIDTH>
__device__ __forceinline__ void store_packed_fields(uint8_t *dst, uint32_t value, int nvalid)
{
    static_assert(WIDTH >= 4 && WIDTH <= 28, "a byte spans at most three fields");
    constexpr int NF = 64 / G;
    constexpr int kRounds = (((NF * WIDTH) >> 3) + 63) >> 6;
    const int lane = (int)(threadIdx.x & 63);
    const int nbytes = (nvalid * WIDTH + 7) >> 3;
#pragma unroll
    for (int t = 0; t < kRounds; ++t) {
        const int j = lane + 64 * t;
        const int f0 = (8 * j) / WIDTH, off = 8 * j - f0 * WIDTH;
        uint32_t bits = 0;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const int f = f0 + k;
            const uint32_t v = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * min(f, NF - 1) * G, (int)value);
            const int sh = k * WIDTH - off;                   // negative only for k == 0
            if (f < NF && sh < 8) bits |= sh >= 0 ? v << sh : v >> -sh;
        }
        if (j < nbytes) dst[j] = (uint8_t)bits;
    }
}

// Calls fn(std::integral_constant<int, s>{}) for the narrow scale width s = 4..7 (wave-uniform).
template <class Fn>
__device__ __forceinline__ void with_scale_width(int sbits, Fn fn)
{
    switch (sbits) {
    case 4: fn(std::integral_constant<int, 4>{}); break;
    case 5: fn(std::integral_constant<int, 5>{}); break;
    case 6: fn(std::integral_constant<int, 6>{}); break;
    default: fn(std::integral_constant<int, 7>{}); break;
    }
}

// The quantize kernels' form of the same store, for all U steps of a wave at once and a scale
// width known at compile time (the division below folds into a multiply): the wave's U * 64/G
// fields of WIDTH bits (4..7) are consecutive in the stream; the field of step u, block k is held
// by lane k*G in byte u of `value` (0 for fields past `nvalid`).  Every lane of the wave must call
// this.
template <int G, int U, int WIDTH>
__device__ __forceinline__ void store_packed_steps(uint8_t *dst, uint32_t value, int nvalid)
{
    static_assert(U <= 4 && WIDTH >= 4 && WIDTH <= 7, "one byte per step in a dword; a byte spans <= 3 fields");
    constexpr int NF = 64 / G, NT = U * NF;
    constexpr int kRounds = (((NT * WIDTH) >> 3) + 63) >> 6;
    const int lane = (int)(threadIdx.x & 63);
    const int nbytes = (nvalid * WIDTH + 7) >> 3;
#pragma unroll
    for (int t = 0; t < kRounds; ++t) {
        const int j = lane + 64 * t;
        const int f0 = (8 * j) / WIDTH, off = 8 * j - f0 * WIDTH;
        uint32_t bits = 0;
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            const int f = f0 + k;
            const int fc = min(f, NT - 1);
            uint32_t v = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * (fc % NF) * G, (int)value);
            v = (v >> (8 * (fc / NF))) & 0xFFu;
            const int sh = k * WIDTH - off;                   // negative only for k == 0
            if (f < NT && sh < 8) bits |= sh >= 0 ? v << sh : v >> -sh;
        }
        if (j < nbytes) dst[j] = (uint8_t)bits;
    }
}

// `nbits` (<= 28) bits starting at bit `bitpos` of a byte array of `total` bytes.
__device__ __forceinline__ uint32_t load_bits(const uint8_t *base, size_t bitpos, int nbits, size_t total)
{
    const size_t byte = bitpos >> 3;
    const int sh = (int)(bitpos & 7);
    uint64_t w = 0;
#pragma unroll
    for (int k = 0; k < 5; ++k)
        if (8 * k < sh + nbits && byte + k < total) w |= (uint64_t)base[byte + k] << (8 * k);
    return (uint32_t)(w >> sh) & ((1u << nbits) - 1u);
}

}  // namespace mxc
