// The quantize kernels of the mxc library (bf16 or binary32 input -> packed codes and scales).
#pragma once

#include "mxc_common.hpp"

namespace mxc {

// ---------------------------------------------------------------------------------------------
// Quantize (Method, "Communication Compression": block-wise quantization, shared exponent).

struct QuantArgs {
    const void *x[32];
    void *codes[32];
    void *scales[32];
    size_t units;       // elements / 8 of one tensor
    ScaleFmt sf;
};

// Eight elements -> packed codes, integer path.  w: the unit's raw input dwords.
template <class E, bool SRC32>
__device__ __forceinline__ uint64_t encode_unit_generic(const u32x4 (&w)[SRC32 ? 2 : 1], int neg_e)
{
    uint64_t packed = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t mag, bits;
        if (SRC32) {
            bits = w[j >> 2][j & 3];
            mag = round_full_sig<E>(__uint_as_float(bits), neg_e);
        } else {
            const uint32_t pair = w[0][j >> 1];
            bits = (j & 1) ? (pair & 0xFFFF0000u) : (pair << 16);
            mag = round_small_sig<E>(__uint_as_float(bits), neg_e + E::beta - 127);
        }
        const uint32_t code = mag | ((bits >> 31) << (E::x + E::y));
        packed |= (uint64_t)code << (j * E::bits);
    }
    return packed;
}

// Eight elements -> packed codes for a one-bit exponent (E1My, the INT grids of the Method list):
// the magnitudes are the uniform grid 0, step, 2 step, ... with step = 2^(1-y), so the code is
// round-half-even(|v| * 2^-e / step), saturated; one multiply by a power of two (exact, or
// so far below half a step that it rounds to zero either way), one round, one clamp.
// inv_step = 2^(-e - 1 + y).
template <class E, bool SRC32>
__device__ __forceinline__ uint64_t encode_unit_uniform(const u32x4 (&w)[SRC32 ? 2 : 1], float inv_step)
{
    static_assert(E::x == 1, "uniform grid: one exponent bit");
    uint64_t packed = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t bits;
        if (SRC32) {
            bits = w[j >> 2][j & 3];
        } else {
            const uint32_t pair = w[0][j >> 1];
            bits = (j & 1) ? (pair & 0xFFFF0000u) : (pair << 16);
        }
        const float q = __builtin_fminf(__builtin_rintf(__builtin_fabsf(__uint_as_float(bits)) * inv_step),
                                        (float)E::magmask);
        const uint32_t code = (uint32_t)q | ((bits >> 31) << (E::x + E::y));
        packed |= (uint64_t)code << (j * E::bits);
    }
    return packed;
}

// Scaled conversions need their byte / word selector as a literal: one wrapper per selector.
template <int K, bool SRC32, int NW>
__device__ __forceinline__ uint32_t cvt_pair_to_fp4(uint32_t old, const u32x4 (&w)[NW], float s)
{
    if (SRC32)
        return __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(old, __uint_as_float(w[K >> 1][2 * (K & 1)]),
                                                        __uint_as_float(w[K >> 1][2 * (K & 1) + 1]), s, K);
    else
        return __builtin_amdgcn_cvt_scalef32_pk_fp4_bf16(old, as_bf16x2(w[0][K]), s, K);
}

// Element pair P (0..3) of the unit -> two bytes in word (P & 1) of `old`.
template <int HWK, int P, bool SRC32, int NW>
__device__ __forceinline__ i16x2 cvt_pair_to_8bit(i16x2 old, const u32x4 (&w)[NW], float s)
{
    constexpr bool hi = (P & 1) != 0;
    if (SRC32) {
        const float a = __uint_as_float(w[P >> 1][2 * (P & 1)]);
        const float b = __uint_as_float(w[P >> 1][2 * (P & 1) + 1]);
        return HWK == HW_BF8 ? __builtin_amdgcn_cvt_scalef32_pk_bf8_f32(old, a, b, s, hi)
                             : __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(old, a, b, s, hi);
    } else {
        const bf16x2 v = as_bf16x2(w[0][P]);
        return HWK == HW_BF8 ? __builtin_amdgcn_cvt_scalef32_pk_bf8_bf16(old, v, s, hi)
                             : __builtin_amdgcn_cvt_scalef32_pk_fp8_bf16(old, v, s, hi);
    }
}

// Four bytes sign<<7 | magnitude (magnitude <= magmask + 1) -> four b-bit codes, squeezed.
template <class E>
__device__ __forceinline__ uint32_t bytes_to_codes(uint32_t v)
{
    // the scale rule keeps |p| below 2^(emax+1); rounding can reach exactly that value, whose
    // code is magmask+1: fold it back onto the largest magnitude
    v -= (v >> (E::x + E::y)) & 0x01010101u;
    // sign from bit 7 down to bit x+y
    v = (v & (E::magmask * 0x01010101u)) |
        ((v >> (7 - E::x - E::y)) & ((E::magmask + 1u) * 0x01010101u));
    return squeeze4<E::bits>(v);
}

// Eight elements -> packed codes with the scaled-conversion instructions.  hw_scale is the
// binary32 whose exponent field is the power of two the inputs are divided by.
template <class E, bool SRC32>
__device__ __forceinline__ uint64_t encode_unit_hw(const u32x4 (&w)[SRC32 ? 2 : 1], float hw_scale)
{
    constexpr int NW = SRC32 ? 2 : 1;
    if (E::hw == HW_FP4) {
        uint32_t r = 0;
        r = cvt_pair_to_fp4<0, SRC32, NW>(r, w, hw_scale);
        r = cvt_pair_to_fp4<1, SRC32, NW>(r, w, hw_scale);
        r = cvt_pair_to_fp4<2, SRC32, NW>(r, w, hw_scale);
        r = cvt_pair_to_fp4<3, SRC32, NW>(r, w, hw_scale);
        return r;
    } else {
        constexpr int K = E::hw == HW_BF8 ? HW_BF8 : HW_FP8;
        i16x2 lo = {0, 0}, hi = {0, 0};
        lo = cvt_pair_to_8bit<K, 0, SRC32, NW>(lo, w, hw_scale);
        lo = cvt_pair_to_8bit<K, 1, SRC32, NW>(lo, w, hw_scale);
        hi = cvt_pair_to_8bit<K, 2, SRC32, NW>(hi, w, hw_scale);
        hi = cvt_pair_to_8bit<K, 3, SRC32, NW>(hi, w, hw_scale);
        const uint32_t c0 = bytes_to_codes<E>(__builtin_bit_cast(uint32_t, lo));
        const uint32_t c1 = bytes_to_codes<E>(__builtin_bit_cast(uint32_t, hi));
        return (uint64_t)c0 | ((uint64_t)c1 << (4 * E::bits));
    }
}

// Shared exponent of a block from the biased exponent field of its maximum, and the unit's eight
// packed codes.  Returns the scale byte in *scale_byte.
template <class E, bool SRC32, bool HW>
__device__ __forceinline__ uint64_t encode_unit(const u32x4 (&w)[SRC32 ? 2 : 1], int expfield,
                                                const ScaleFmt &sf, int *scale_byte)
{
    constexpr bool kHw = HW && E::hw != HW_NONE;
    // shared exponent: floor(log2 max) - emax, as a scale code, clamped to the scale format
    const int unclamped = expfield - 127 - E::emax + sf.sbias;
    const bool finite = expfield != 255;
    const int sc = finite ? min(max(unclamped, 0), sf.smax) : sf.nonfinite;
    const int e = sc - sf.sbias;
    *scale_byte = sc;

    uint64_t packed;
    if constexpr (kHw) {
        // divide by 2^(e - beta + hw_bias): the element format's smallest normal then falls on
        // the hardware format's smallest normal.  Usable while that power of two has a binary32
        // exponent field and (for the 8-bit formats) the scale's upper clamp is idle, which is
        // what bounds |p| below 2^(emax+1).
        const int field = e - E::beta + E::hw_bias + 127;
        const bool ok = field >= 0 && field <= 254 && (E::hw == HW_FP4 || unclamped <= sf.smax);
        if (__builtin_amdgcn_ballot_w64(!ok && finite) == 0) {
            packed = encode_unit_hw<E, SRC32>(w, __uint_as_float((uint32_t)max(field, 0) << 23));
        } else {
            packed = encode_unit_generic<E, SRC32>(w, -e);
        }
    } else if constexpr (E::x == 1) {
        // 2^(-e - 1 + y) as a binary32: its exponent field is in range for every scale a finite
        // block can have (e <= 126), checked all the same
        const int field = -e - 1 + E::y + 127;
        if (__builtin_amdgcn_ballot_w64((field < 1 || field > 254) && finite) == 0) {
            packed = encode_unit_uniform<E, SRC32>(w, __uint_as_float((uint32_t)min(max(field, 1), 254) << 23));
        } else {
            packed = encode_unit_generic<E, SRC32>(w, -e);
        }
    } else {
        packed = encode_unit_generic<E, SRC32>(w, -e);
    }
    return finite ? packed : 0;
}

// SRC32 = false: bfloat16 input, one 128-bit load per unit.
// SRC32 = true : binary32 input, two 128-bit loads per unit.
// U: units per lane.  NTL/NTS: nontemporal loads / stores.  HW: use scaled conversions.
// XPOSE (binary32 input only): load the wave's 32-byte units as contiguous 16-byte pieces and
// hand each lane its unit through a wave-private LDS tile, instead of two 16-byte loads per lane
// that each use half of every cache line they touch.
template <class E, int B, bool SRC32, int U, bool NTL, bool NTS, bool HW, bool XPOSE = false>
__global__ __launch_bounds__(kThreads) void quantize_kernel(QuantArgs a)
{
    constexpr int G = B / 8;                     // lanes per block
    constexpr int NW = SRC32 ? 2 : 1;
    const int lane = (int)(threadIdx.x & 63);
    const int wave = (int)(threadIdx.x >> 6);
    const size_t wave_base =
        ((size_t)blockIdx.x * (kThreads / 64) + (size_t)wave) * (size_t)(U * 64);
    const void *xin = a.x[blockIdx.y];
    uint32_t *codes = (uint32_t *)a.codes[blockIdx.y];
    uint8_t *scales = (uint8_t *)a.scales[blockIdx.y];
    const ScaleFmt sf = a.sf;

    u32x4 w[U][NW];
    bool valid[U];
    if (XPOSE && SRC32) {
        __shared__ u32x4 xtile[kThreads / 64][XPOSE ? U * 64 * 2 : 1];
        u32x4 *t = xtile[wave];
        const u32x4 *src = (const u32x4 *)xin + wave_base * 2;       // 2 pieces per unit
        const size_t pieces_left = wave_base < a.units ? (a.units - wave_base) * 2 : 0;
        u32x4 pv[U * 2];
#pragma unroll
        for (int k = 0; k < U * 2; ++k) {
            const int piece = k * 64 + lane;
            pv[k] = (size_t)piece < pieces_left ? ld<NTL>(src + piece) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int k = 0; k < U * 2; ++k) t[k * 64 + lane] = pv[k];
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t unit = wave_base + (size_t)(u * 64 + lane);
            valid[u] = unit < a.units;
            w[u][0] = t[(u * 64 + lane) * 2];
            w[u][NW - 1] = t[(u * 64 + lane) * 2 + 1];
        }
    } else {
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t unit = wave_base + (size_t)(u * 64 + lane);
        valid[u] = unit < a.units;
        const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int h = 0; h < NW; ++h)
            w[u][h] = valid[u] ? ld<NTL>((const u32x4 *)xin + unit * NW + h) : zero;
    }
    }

    int my_scale = 0;                            // the scale byte this lane will store
    uint32_t narrow_scales = 0;                  // narrow scale codes of this lane's blocks, step u in byte u
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t unit = wave_base + (size_t)(u * 64 + lane);
        int expfield;                            // biased exponent field of the block maximum
        if (SRC32) {
            uint32_t m = 0;
#pragma unroll
            for (int h = 0; h < NW; ++h)
#pragma unroll
                for (int j = 0; j < 4; ++j) m = max(m, w[u][h][j] & 0x7FFFFFFFu);
            expfield = (int)(block_max<B>(m) >> 23);
        } else {
            const u32x4 v = w[u][0];
            uint32_t m = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                                    pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
            m = max(m & 0xFFFFu, m >> 16);
            expfield = (int)(block_max<B>(m) >> 7);
        }
        int sc;
        const uint64_t packed = encode_unit<E, SRC32, HW>(w[u], expfield, sf, &sc);
        store_codes<E::bits, NTS>(codes, unit, packed, a.units);

        // Every lane of a block knows the block's scale.
        if (sf.sbits < 8) {
            // packed scale stream: stored for all steps at once below
            if (valid[u]) narrow_scales |= (uint32_t)sc << (8 * u);
        } else if (U % G == 0) {
            // Over G consecutive steps lane l keeps the scale of step (l % G); after the G-th
            // step each lane stores one byte, so the wave writes 64 consecutive scale bytes.
            if ((lane & (G - 1)) == (u & (G - 1))) my_scale = sc;
            if ((u & (G - 1)) == G - 1) {
                const int step = u - (G - 1) + (lane & (G - 1));
                const size_t first_unit = wave_base + (size_t)(step * 64 + (lane / G) * G);
                if (first_unit < a.units) scales[first_unit / G] = (uint8_t)my_scale;
            }
        } else {
            if ((lane & (G - 1)) == 0 && valid[u]) scales[unit / G] = (uint8_t)sc;
        }
    }
    if (sf.sbits < 8 && wave_base < a.units) {
        // the wave's U * 64/G scale fields are a byte-aligned run of the stream
        const size_t first_block = wave_base / G;
        const size_t left = a.units / G - first_block;
        const int nvalid = (int)(left < (size_t)(U * 64 / G) ? left : (size_t)(U * 64 / G));
        uint8_t *run = scales + ((first_block * (size_t)sf.sbits) >> 3);
        with_scale_width(sf.sbits, [&](auto w) { store_packed_steps<G, U, decltype(w)::value>(run, narrow_scales, nvalid); });
    }
}

}  // namespace mxc
