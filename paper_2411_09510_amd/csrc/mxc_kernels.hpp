// Device code of the mxc library for gfx950 (wave64).
//
// Work decomposition shared by all kernels: a tensor [tokens x hidden] is treated as a flat
// array (blocks never straddle rows because hidden % block == 0, and rows are packed back to
// back, so the flat view of inputs, packed codes and scales is exact).  A "unit" is 8 consecutive
// elements: one 128-bit load of bf16, one dword of 4-bit codes, b bytes of b-bit codes.  A block of
// B elements is B/8 neighbouring lanes of one wave (1, 2 or 4 lanes), so the block maximum is a
// quad-local DPP reduction and never touches LDS.  Each wave owns kUnitsPerLane * 64 consecutive
// units; in step u lane l handles unit (wave_base + u*64 + l), which keeps every load and store
// instruction contiguous across the wave.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mxc {

constexpr int kThreads = 256;        // 4 waves per workgroup
constexpr int kUnitsPerLane = 4;     // 16-byte units per lane and tile
constexpr int kUnitsPerWave = 64 * kUnitsPerLane;
constexpr int kUnitsPerGroup = kThreads * kUnitsPerLane;

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Element format ExMy (Method, parameter list): facts derived at compile time.
template <int X, int Y>
struct Elem {
    static constexpr int x = X, y = Y;
    static constexpr int bits = 1 + X + Y;
    static constexpr int beta = (1 << (X - 1)) - 1;
    static constexpr int emax = (1 << X) - 1 - beta;
    static constexpr uint32_t magmask = (1u << (X + Y)) - 1u;
};

// Scale format EsM0, runtime (s only changes two clamps per block).
struct ScaleFmt {
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

// Maximum over the B/8 lanes that share a block.
template <int B>
__device__ __forceinline__ uint32_t block_max(uint32_t m)
{
    if (B >= 16) m = max(m, dpp<quad_perm(1, 0, 3, 2)>(m));
    if (B >= 32) m = max(m, dpp<quad_perm(2, 3, 0, 1)>(m));
    return m;
}

// Scale byte from the block maximum's biased binary32/bfloat16 exponent field (0..255):
// floor(log2 max) - emax + sbias, clamped; 255 in the exponent field means Inf/NaN.
template <class E>
__device__ __forceinline__ int scale_code(int max_expfield, const ScaleFmt &sf)
{
    int c = max_expfield - 127 - E::emax + sf.sbias;
    c = min(max(c, 0), sf.smax);
    return max_expfield == 255 ? sf.nonfinite : c;
}

// ---------------------------------------------------------------------------------------------
// Rounding of one element to an ExMy magnitude code, ties to the even code, saturating.
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
// Moving b-bit codes between "8 codes per lane" and the packed little-endian bit stream.
// A quad of lanes owns 32 codes = b dwords of the stream, at dword index quad*b.

// Store: lane holds its 8 codes in the low 8b bits of v.
template <int BITS>
__device__ __forceinline__ void store_codes(uint32_t *codes, size_t unit, uint64_t v, bool valid)
{
    const int i = (int)(threadIdx.x & 3);
    uint32_t *q = codes + (unit >> 2) * BITS;
    if (BITS == 4) {
        if (valid) codes[unit] = (uint32_t)v;
    } else if (BITS == 5) {
        // lane i's 40 bits start at stream bit 40i = dword i, bit 8i
        uint64_t w = v << (8 * i);
        uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
        uint32_t from_prev = dpp<quad_perm(3, 0, 1, 2)>(hi);     // lane i gets hi of lane i-1
        uint32_t d = lo | (i ? from_prev : 0u);
        if (valid) {
            q[i] = d;
            if (i == 0) q[4] = from_prev;                        // hi of lane 3
        }
    } else if (BITS == 6) {
        // pairs of lanes own 3 dwords: even lane bits 0..47, odd lane bits 48..95
        uint64_t w = v << (16 * (i & 1));
        uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
        uint32_t give = (i & 1) ? lo : hi;
        uint32_t got = dpp<quad_perm(1, 0, 3, 2)>(give);          // odd lane gets even's hi
        uint32_t *p = q + 3 * (i >> 1);
        if (valid) {
            if (i & 1) {
                p[1] = lo | got;
                p[2] = hi;
            } else {
                p[0] = lo;
            }
        }
    } else {  // BITS == 3: lane i's 24 bits start at stream bit 24i
        const int s = (32 - 8 * i) & 31;                          // 0, 24, 16, 8
        uint64_t w = v << s;
        uint32_t lo = (uint32_t)w, hi = (uint32_t)(w >> 32);
        uint32_t from_next = dpp<quad_perm(1, 2, 3, 3)>(lo);      // lane i gets lo of lane i+1
        uint32_t d = (i ? hi : lo) | from_next;
        if (valid && i < 3) q[i] = d;
    }
}

// Load: returns the lane's 8 codes in the low 8b bits.
template <int BITS>
__device__ __forceinline__ uint64_t load_codes(const uint32_t *codes, size_t unit, bool valid)
{
    const int i = (int)(threadIdx.x & 3);
    const uint32_t *q = codes + (unit >> 2) * BITS;
    if (BITS == 4) {
        return valid ? codes[unit] : 0u;
    } else if (BITS == 5) {
        uint32_t d = 0, extra = 0;
        if (valid) {
            d = q[i];
            if (i == 0) extra = q[4];
        }
        uint32_t give = i ? d : extra;
        uint32_t next = dpp<quad_perm(1, 2, 3, 0)>(give);         // lane i gets dword i+1
        uint64_t w = ((uint64_t)next << 32) | d;
        return (w >> (8 * i)) & ((1ull << 40) - 1);
    } else if (BITS == 6) {
        const uint32_t *p = q + 3 * (i >> 1);
        uint32_t a = 0, b = 0;
        if (valid) {
            if (i & 1) {
                a = p[1];
                b = p[2];
            } else {
                a = p[0];
            }
        }
        uint32_t other = dpp<quad_perm(1, 0, 3, 2)>(a);           // even lane gets dword 1
        uint64_t even = (uint64_t)a | ((uint64_t)(other & 0xFFFFu) << 32);
        uint64_t odd = (uint64_t)(a >> 16) | ((uint64_t)b << 16);
        return (i & 1) ? odd : even;
    } else {  // BITS == 3
        uint32_t d = 0;
        if (valid && i < 3) d = q[i];
        uint32_t prev = dpp<quad_perm(0, 0, 1, 2)>(d);            // lane i gets dword i-1
        uint64_t w = ((uint64_t)d << 32) | prev;
        return (w >> (32 - 8 * i)) & 0xFFFFFFull;
    }
}

// ---------------------------------------------------------------------------------------------
// Quantize (Method, "Communication Compression": block-wise quantization, shared exponent).

struct QuantArgs {
    const void *x[32];
    void *codes[32];
    void *scales[32];
    size_t units;       // elements / 8 of one tensor
    ScaleFmt sf;
};

// SRC32 = false: bfloat16 input, one 128-bit load per unit.
// SRC32 = true : binary32 input, two 128-bit loads per unit.
template <class E, int B, bool SRC32>
__global__ __launch_bounds__(kThreads) void quantize_kernel(QuantArgs a)
{
    constexpr int G = B / 8;                     // lanes per block
    const int lane = (int)(threadIdx.x & 63);
    const int wave = (int)(threadIdx.x >> 6);
    const size_t wave_base =
        ((size_t)blockIdx.x * (kThreads / 64) + (size_t)wave) * (size_t)kUnitsPerWave;
    const void *xin = a.x[blockIdx.y];
    uint32_t *codes = (uint32_t *)a.codes[blockIdx.y];
    uint8_t *scales = (uint8_t *)a.scales[blockIdx.y];
    const ScaleFmt sf = a.sf;

    u32x4 w[kUnitsPerLane][SRC32 ? 2 : 1];
    bool valid[kUnitsPerLane];
#pragma unroll
    for (int u = 0; u < kUnitsPerLane; ++u) {
        const size_t unit = wave_base + (size_t)(u * 64 + lane);
        valid[u] = unit < a.units;
        const u32x4 zero = {0u, 0u, 0u, 0u};
        if (SRC32) {
            const u32x4 *p = (const u32x4 *)xin + unit * 2;
            w[u][0] = valid[u] ? p[0] : zero;
            w[u][SRC32 ? 1 : 0] = valid[u] ? p[1] : zero;
        } else {
            w[u][0] = valid[u] ? ((const u32x4 *)xin)[unit] : zero;
        }
    }

    int my_scale = 0;                            // the scale byte this lane will store
#pragma unroll
    for (int u = 0; u < kUnitsPerLane; ++u) {
        const size_t unit = wave_base + (size_t)(u * 64 + lane);
        int expfield;
        if (SRC32) {
            uint32_t m = 0;
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int j = 0; j < 4; ++j) m = max(m, w[u][h][j] & 0x7FFFFFFFu);
            m = block_max<B>(m);
            expfield = (int)(m >> 23);
        } else {
            const u32x4 v = w[u][0];
            uint32_t m = pk_max_u16(pk_max_u16(v.x & 0x7FFF7FFFu, v.y & 0x7FFF7FFFu),
                                    pk_max_u16(v.z & 0x7FFF7FFFu, v.w & 0x7FFF7FFFu));
            m = max(m & 0xFFFFu, m >> 16);
            m = block_max<B>(m);
            expfield = (int)(m >> 7);
        }
        const int sc = scale_code<E>(expfield, sf);
        const bool finite = expfield != 255;
        const int neg_e = sf.sbias - sc;         // -e

        uint64_t packed = 0;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t mag, sign;
            if (SRC32) {
                const uint32_t bits = w[u][j >> 2][j & 3];
                mag = round_full_sig<E>(__uint_as_float(bits), neg_e);
                sign = bits >> 31;
            } else {
                const uint32_t pair = w[u][0][j >> 1];
                const uint32_t bits = (j & 1) ? (pair & 0xFFFF0000u) : (pair << 16);
                mag = round_small_sig<E>(__uint_as_float(bits), neg_e + E::beta - 127);
                sign = bits >> 31;
            }
            const uint32_t code = finite ? (mag | (sign << (E::x + E::y))) : 0u;
            packed |= (uint64_t)code << (j * E::bits);
        }
        store_codes<E::bits>(codes, unit, packed, valid[u]);

        // Every lane of a block knows the block's scale.  Over G consecutive steps lane l keeps
        // the scale of step (l % G); after the G-th step each lane stores one byte, so that the
        // wave writes 64 consecutive scale bytes with one instruction.
        if ((lane & (G - 1)) == (u & (G - 1))) my_scale = sc;
        if ((u & (G - 1)) == G - 1) {
            const int step = u - (G - 1) + (lane & (G - 1));
            const size_t first_unit = wave_base + (size_t)(step * 64 + (lane / G) * G);
            if (first_unit < a.units) scales[first_unit / G] = (uint8_t)my_scale;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Dequantize + reduce (Profiling: decompress the gathered partials, then a plain sum).

struct ReduceArgs {
    const void *codes[32];
    const void *scales[32];
    void *out;
    size_t units;
    int tp;
    ScaleFmt sf;
};

// Decode code j of `v` to binary32 times 2^k (exact): the magnitude code, shifted so that its
// mantissa sits at the top of binary32's fraction field, is value * 2^(beta-127) as a (possibly
// subnormal) binary32; ldexp moves it to value * 2^e.
template <class E>
__device__ __forceinline__ float decode(uint64_t v, int j, int k /* e + 127 - beta */)
{
    const uint32_t c = (uint32_t)(v >> (j * E::bits));
    const uint32_t bits = ((c & E::magmask) << (23 - E::y)) | ((c >> (E::x + E::y)) << 31);
    return ldexpf(__uint_as_float(bits), k);
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    uint32_t r = (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
    return (f != f) ? 0x7FC0u : r;
}

template <class E, int B, bool OUT_BF16>
__global__ __launch_bounds__(kThreads) void dequant_reduce_kernel(ReduceArgs a)
{
    constexpr int G = B / 8;
    constexpr int RC = 8;                        // ranks loaded together
    const int lane = (int)(threadIdx.x & 63);
    const int wave = (int)(threadIdx.x >> 6);
    const size_t wave_base =
        ((size_t)blockIdx.x * (kThreads / 64) + (size_t)wave) * (size_t)kUnitsPerWave;
    const ScaleFmt sf = a.sf;

    for (int u = 0; u < kUnitsPerLane; ++u) {
        const size_t unit = wave_base + (size_t)(u * 64 + lane);
        const bool valid = unit < a.units;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        bool poisoned = false;                   // some rank marked this block non-finite
        for (int r0 = 0; r0 < a.tp; r0 += RC) {
            uint64_t v[RC];
            int sc[RC];
#pragma unroll
            for (int i = 0; i < RC; ++i) {
                const bool on = valid && (r0 + i < a.tp);
                const int r = min(r0 + i, a.tp - 1);
                v[i] = load_codes<E::bits>((const uint32_t *)a.codes[r], unit, on);
                sc[i] = on ? (int)((const uint8_t *)a.scales[r])[unit / G] : 0;
            }
#pragma unroll
            for (int i = 0; i < RC; ++i) {
                if (r0 + i < a.tp) {
                    const int k = sc[i] - sf.sbias + 127 - E::beta;
                    poisoned = poisoned || (sf.has_nan && sc[i] == 255);
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        const float d = decode<E>(v[i], j, k);
                        acc[j] = (r0 + i == 0) ? d : acc[j] + d;
                    }
                }
            }
        }
        if (poisoned) {
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] = __uint_as_float(0x7FC00000u);
        }
        if (valid) {
            if (OUT_BF16) {
                u32x4 o;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    o[j] = f32_to_bf16_rne(acc[2 * j]) | (f32_to_bf16_rne(acc[2 * j + 1]) << 16);
                ((u32x4 *)a.out)[unit] = o;
            } else {
                f32x4 *o = (f32x4 *)a.out + unit * 2;
                o[0] = f32x4{acc[0], acc[1], acc[2], acc[3]};
                o[1] = f32x4{acc[4], acc[5], acc[6], acc[7]};
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Plain 128-bit copy, the practical bandwidth ceiling the codec kernels are compared with.
__global__ __launch_bounds__(kThreads) void copy_kernel(u32x4 *dst, const u32x4 *src, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * (size_t)kUnitsPerGroup + threadIdx.x;
    u32x4 v[kUnitsPerLane];
#pragma unroll
    for (int u = 0; u < kUnitsPerLane; ++u) {
        const size_t i = base + (size_t)u * kThreads;
        if (i < n16) v[u] = src[i];
    }
#pragma unroll
    for (int u = 0; u < kUnitsPerLane; ++u) {
        const size_t i = base + (size_t)u * kThreads;
        if (i < n16) dst[i] = v[u];
    }
}

}  // namespace mxc
