// The dequantize + reduce kernels of the mxc library: tile form, half-chunk form, their fused
// (re-quantizing) and own-raw variants.
#pragma once

#include "mxc_quantize.hpp"   // the fused form quantizes its sums with the quantizer's encode step

namespace mxc {

// ---------------------------------------------------------------------------------------------
// Arguments and decoding helpers of the dequantize + reduce kernel.

struct ReduceArgs {
    const void *codes[32];
    const void *scales[32];
    void *out;          // reduced tensor, or NULL for the fused form
    void *codes_out;    // fused form: packed codes of the re-quantized sum
    void *scales_out;   // fused form: its scale bytes
    const void *own_x;  // OWN form: this rank's uncompressed bf16 partial
    int own_rank;       // OWN form: the rank whose term is read from own_x, else -1
    size_t units;
    int tp;
    ScaleFmt sf;
};

// The accumulators start at -0.0: x + (-0.0) is x for every x (including +0, -0 and NaN), so
// adding rank 0's value to it is the same as starting the fold from that value.
constexpr float kFoldStart = -0.0f;

// Adds eight bfloat16 values, given as four dwords, to acc.
__device__ __forceinline__ void add_raw_bf16(const u32x4 v, float *acc)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        acc[2 * j] += __uint_as_float(v[j] << 16);
        acc[2 * j + 1] += __uint_as_float(v[j] & 0xFFFF0000u);
    }
}

template <int K>
__device__ __forceinline__ f32x2 cvt_fp4_pair(uint32_t v, float s)
{
    return __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(v, s, K);
}

template <int HWK, bool HI>
__device__ __forceinline__ f32x2 cvt_8bit_pair(uint32_t v, float s)
{
    return HWK == HW_BF8 ? __builtin_amdgcn_cvt_scalef32_pk_f32_bf8(v, s, HI)
                         : __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(v, s, HI);
}

// (a & m) | (b & ~m): one v_bfi / v_bitop3.
__device__ __forceinline__ uint32_t bitselect(uint32_t m, uint32_t a, uint32_t b)
{
    return (a & m) | (b & ~m);
}

// Four b-bit codes in the low 4b bits of f (bits above are ignored) -> four bytes
// sign<<7 | magnitude << E::dec_pad (the byte the format's hardware decode format expects).
//
// General form: copy k of f, shifted left by k*(8-b), carries code k's magnitude at byte k and
// code k-1's sign at bit 7 of byte k-1; four selects stitch the copies together and one mask
// clears what lies between magnitude and sign.
//
// 5-bit codes take fewer instructions with two 24-bit multiplies, each of which makes two shifted
// copies at once: codes 0 and 2 (bits 0-4, 10-14) times 1 + 2^6 puts them at bits 0 and 16, codes
// 1 and 3 (bits 5-9, 15-19) times 2^3 + 2^9 puts them at bits 8 and 24.  The unwanted cross
// products land between the wanted fields (bits 6-15 and 14-23, carries included) and are dropped
// by the byte permute and the masks that follow.
template <class E>
__device__ __forceinline__ uint32_t codes_to_bytes(uint32_t f)
{
    constexpr int b = E::bits, g = 8 - E::bits;
    if (b == 5) {
        const uint32_t even = __umul24(f & 0x07C1Fu, (1u << 6) + 1u);
        const uint32_t odd = __umul24(f & 0xF83E0u, (1u << 9) + (1u << 3));
        // bytes 0 and 2 of `even`, bytes 1 and 3 of `odd`: code k in bits 0-4 of byte k (a byte
        // permute, which the compiler keeps as one instruction; an and/or select it splits up)
        const uint32_t c5 = __builtin_amdgcn_perm(odd, even, 0x07020500u);
        // (a one-mantissa-bit format's magnitude moves up by its pad bit: see below)
        return ((c5 & 0x0F0F0F0Fu) << E::dec_pad) | ((c5 << 3) & 0x80808080u);
    }
    uint32_t r = f;
    r = bitselect((1u << (b - 1)) - 1u, r, f << g);
    r = bitselect((1u << (8 + b - 1)) - 1u, r, f << (2 * g));
    r = bitselect((1u << (16 + b - 1)) - 1u, r, f << (3 * g));
    r = bitselect((1u << (24 + b - 1)) - 1u, r, f << (4 * g));
    r &= (E::magmask | 0x80u) * 0x01010101u;
    // one-mantissa-bit formats: the magnitude moves up by the pad bit, the sign stays
    if (E::dec_pad) r = (r & 0x80808080u) | ((r & 0x7F7F7F7Fu) << E::dec_pad);
    return r;
}

// Eight codes -> eight binary32 values times the power of two in hw_scale's exponent field.
template <class E>
__device__ __forceinline__ void decode_unit_hw(uint64_t v, float hw_scale, float (&d)[8])
{
    f32x2 r0, r1, r2, r3;
    if (E::hw_dec == HW_FP4) {
        r0 = cvt_fp4_pair<0>((uint32_t)v, hw_scale);
        r1 = cvt_fp4_pair<1>((uint32_t)v, hw_scale);
        r2 = cvt_fp4_pair<2>((uint32_t)v, hw_scale);
        r3 = cvt_fp4_pair<3>((uint32_t)v, hw_scale);
    } else {
        constexpr int K = E::hw_dec == HW_BF8 ? HW_BF8 : HW_FP8;
        const uint32_t b0 = codes_to_bytes<E>((uint32_t)v);
        const uint32_t b1 = codes_to_bytes<E>((uint32_t)(v >> (4 * E::bits)));
        r0 = cvt_8bit_pair<K, false>(b0, hw_scale);
        r1 = cvt_8bit_pair<K, true>(b0, hw_scale);
        r2 = cvt_8bit_pair<K, false>(b1, hw_scale);
        r3 = cvt_8bit_pair<K, true>(b1, hw_scale);
    }
    d[0] = r0.x; d[1] = r0.y; d[2] = r1.x; d[3] = r1.y;
    d[4] = r2.x; d[5] = r2.y; d[6] = r3.x; d[7] = r3.y;
}

// Two binary32 values -> two bfloat16 (a in the low half), round to nearest even, NaN -> 0x7FC0.
// The conversion is the compiler's (v_cvt_pk_bf16_f32 on gfx950: round to nearest even, bfloat16
// subnormals kept); it keeps a NaN's sign and payload, so NaN halves, (h & 0x7FFF) > 0x7F80, are
// replaced afterwards: adding 0x7F carries exactly those into bit 15, and a 24-bit multiply
// widens the two flag bits into half-word masks.
__device__ __forceinline__ uint32_t f32x2_to_bf16x2_rne(float a, float b)
{
    const f32x2 v = {a, b};
    const uint32_t r = __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
    const uint32_t t = ((r & 0x7FFF7FFFu) + 0x007F007Fu) & 0x80008000u;
    const uint32_t m = __umul24(t >> 15, 0xFFFFu);
    return bitselect(m, 0x7FC07FC0u, r);
}

// LEN bits starting at bit `pos` of a little-endian stream held in NW dwords.  Callers pass
// positions that are constants after unrolling, so this folds to one or two instructions.
template <int NW>
__device__ __forceinline__ uint32_t stream_bits_rt(const uint32_t (&s)[NW], int pos, int len)
{
    const int wd = pos >> 5, off = pos & 31;
    const uint32_t mask = len >= 32 ? 0xFFFFFFFFu : ((1u << len) - 1u);
    uint32_t v = s[wd] >> off;
    if (off + len > 32) v |= s[wd + 1 < NW ? wd + 1 : wd] << (32 - off);
    return v & mask;
}

// ---------------------------------------------------------------------------------------------
// Dequantize + reduce (Profiling: decompress the gathered partials, then a plain sum).
//
// Each lane owns a "chunk" of 32 consecutive elements (one block of 32, two of 16, four of 8): its
// codes are 4b contiguous bytes per rank, its scales 1, 2 or 4 contiguous bytes per rank.  A wave
// tile is the 64 chunks of one wave: per rank 16*b contiguous 16-byte pieces of codes.  4-bit
// codes are one 128-bit load per lane; 3-, 5- and 6-bit codes, whose per-lane dwords are 12, 20
// or 24 bytes apart, are fetched as the tile's contiguous pieces and redistributed through LDS
// (each load instruction then asks the memory system for whole 128-byte lines; per-lane dword
// loads ask for 64-byte halves and run 5 to 8 % slower).  The lane's 32 sums are exchanged
// through the same wave-private LDS area so that the wave writes its 8 KiB (4 KiB for bf16) of
// output as contiguous 128-bit stores.  A tensor's last chunk may hold only 8, 16 or 24 elements
// (blocks of 8 or 16).

// What a lane fetches for one rank of its chunk: W dwords of codes and the chunk's scale codes,
// one per byte.
template <int W>
struct ChunkBits {
    uint32_t cw[W];
    uint32_t sw;
};

// Loads the lane's share of one rank's arrays for the wave tile that starts at chunk
// `wave_chunk0`.  A lane that is not `on` (past the end, a rank beyond tp, the own rank of the OWN
// form) loads nothing and reads as code 0 with "e = 0".  STAGED: the codes of a full wave tile
// (`full`) are left to request_codes_to_lds and only the scales are loaded here.  `tail_units` is 0
// for a whole chunk; the tensor's last chunk holds only 1 to 3 units of 8 elements when the size
// is not a multiple of 32 (blocks of 8 or 16), and that one lane fetches its bytes one by one so
// that nothing past the arrays is read.  `units` is the tensor's size in units.
// COOP (full tiles with a narrow scale format only): the tile's 64 * NB scale fields are a
// byte-aligned run of 8 * NB * s bytes of the stream; the wave fetches it as dwords, one per lane,
// and c.sw receives this lane's raw dword, from which spread_scale_fields later gives every
// lane its own fields (one load per rank instead of up to five byte loads per lane).
template <class E, int B, bool NTL, bool STAGED = false, bool COOP = false>
__device__ __forceinline__ void load_chunk(ChunkBits<E::bits> &c, const void *codes, const void *scales,
                                           size_t wave_chunk0, int lane, bool on, const ScaleFmt &sf,
                                           size_t units, bool full = false, int tail_units = 0)
{
    constexpr int W = E::bits, NB = 32 / B;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const uint32_t *cp = (const uint32_t *)codes + wave_chunk0 * W + lane * W;
#pragma unroll
    for (int k = 0; k < W; ++k) c.cw[k] = 0u;
    // NB scale bytes, little-endian in one register; idle lanes read as "e = 0"
    uint32_t sb = (uint32_t)sf.sbias * 0x01010101u;
    if (on && tail_units) {
        const uint8_t *bp = (const uint8_t *)cp;
        const int nbytes = tail_units * W;       // a unit's 8 codes are W bytes
#pragma unroll
        for (int k = 0; k < W; ++k)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (4 * k + j < nbytes) c.cw[k] |= (uint32_t)bp[4 * k + j] << (8 * j);
        if (sf.sbits == 8) {
            const uint8_t *sp = (const uint8_t *)scales + wave_chunk0 * NB + lane * NB;
            const int nscales = tail_units * 8 / B;
            sb = 0;
#pragma unroll
            for (int n = 0; n < NB; ++n)
                sb |= (n < nscales ? (uint32_t)sp[n] : (uint32_t)sf.sbias) << (8 * n);
        }
    } else if (on) {
        if (!(STAGED && full)) {
            if (W == 4) {
                const u32x4 v = ld<NTL>((const u32x4 *)cp);
                c.cw[0] = v.x; c.cw[1] = v.y; c.cw[2] = v.z; c.cw[3 < W ? 3 : 0] = v.w;
            } else if (W == 6) {
#pragma unroll
                for (int k = 0; k < 3; ++k) {
                    const u32x2 v = ld<NTL>((const u32x2 *)cp + k);
                    c.cw[(2 * k) < W ? 2 * k : 0] = v.x;
                    c.cw[(2 * k + 1) < W ? 2 * k + 1 : 0] = v.y;
                }
            } else {
#pragma unroll
                for (int k = 0; k < W; ++k) c.cw[k] = ld<NTL>(cp + k);
            }
        }
        if (sf.sbits == 8) {
            const uint8_t *sp = (const uint8_t *)scales + wave_chunk0 * NB + lane * NB;
            if (NB == 1) sb = ld<NTL>(sp);
            else if (NB == 2) sb = ld<NTL>((const uint16_t *)sp);
            else sb = ld<NTL>((const uint32_t *)sp);
        }
    }
    if (COOP) {
        const uint32_t *sp = (const uint32_t *)((const uint8_t *)scales + ((wave_chunk0 * NB * (size_t)sf.sbits) >> 3));
        sb = (on && lane < 2 * NB * sf.sbits) ? ld<NTL>(sp + lane) : 0u;
    } else if (on && sf.sbits < 8) {
        // packed stream: NB fields of s bits, re-spread to one byte each (load_bits reads no
        // byte past the stream's end; fields of blocks past the end are never used)
        const size_t chunk = wave_chunk0 + (size_t)lane;
        const size_t nblocks = units * 8 / B;
        const uint32_t raw = load_bits((const uint8_t *)scales, chunk * NB * (size_t)sf.sbits,
                                       NB * sf.sbits, (nblocks * (size_t)sf.sbits + 7) >> 3);
        sb = 0;
#pragma unroll
        for (int n = 0; n < NB; ++n)
            sb |= ((raw >> (n * sf.sbits)) & ((1u << sf.sbits) - 1u)) << (8 * n);
    }
    c.sw = sb;
}

// Second half of the cooperative scale load: `raw` is the dword this lane fetched of the wave's
// scale-field run (lane k holds dword k).  Returns NB consecutive fields starting at field
// `first` of the run, one per byte.  Every lane of the wave must call this.
template <int NB>
__device__ __forceinline__ uint32_t spread_scale_fields_at(uint32_t raw, int first, int sbits)
{
    const int pos = first * sbits;               // first bit of the wanted fields
    const int d0 = pos >> 5;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * d0, (int)raw);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute(4 * min(d0 + 1, 63), (int)raw);
    const uint32_t bits = (uint32_t)((((uint64_t)hi << 32) | lo) >> (pos & 31));
    uint32_t sb = 0;
#pragma unroll
    for (int n = 0; n < NB; ++n) sb |= ((bits >> (n * sbits)) & ((1u << sbits) - 1u)) << (8 * n);
    return sb;
}

// The tile form's case: the lane's own NB fields.
template <int NB>
__device__ __forceinline__ uint32_t spread_scale_fields(uint32_t raw, int lane, int sbits)
{
    return spread_scale_fields_at<NB>(raw, lane * NB, sbits);
}

// 32 five-bit codes (5 dwords of the bit stream) -> 32 six-bit slots (6 dwords), slot = code << 1.
// Four codes at a time: their 20 bits are taken one position up (bits 1..20), codes 2 and 3 move
// two positions up by adding three times their own bits (low part + 4 * high part), codes 1 and 3
// one more by adding themselves; the resulting 24-bit pieces are whole bytes of the slot stream,
// which three byte permutes per four pieces put together.
__device__ __forceinline__ void widen_5_to_6(const uint32_t (&in)[5], uint32_t (&out)[6])
{
    uint32_t p[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) {
        const int pos = 20 * q - 1;              // stream bit that lands on bit 0 (constant)
        uint32_t x;
        if (q == 0) {
            x = in[0] << 1;
        } else {
            const int wd = pos >> 5, off = pos & 31;
            x = in[wd] >> off;
            if (off + 21 > 32) x |= in[wd + 1 < 5 ? wd + 1 : wd] << (32 - off);
        }
        x &= 0x1FFFFEu;
        const uint32_t t = x & 0x1FF800u;        // codes 2 and 3
        x = __umul24(t, 3u) + x;
        const uint32_t u = x & ((0x1Fu << 6) | (0x1Fu << 18));   // codes 1 and 3
        p[q] = x + u;
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        out[3 * k + 0] = __builtin_amdgcn_perm(p[4 * k + 1], p[4 * k + 0], 0x04020100u);
        out[3 * k + 1] = __builtin_amdgcn_perm(p[4 * k + 2], p[4 * k + 1], 0x05040201u);
        out[3 * k + 2] = __builtin_amdgcn_perm(p[4 * k + 3], p[4 * k + 2], 0x06050402u);
    }
}

// Decodes one rank's chunk and adds it to the lane's 32 sums; notes blocks marked non-finite.
template <class E, int B, bool HW>
__device__ __forceinline__ void add_chunk(const ChunkBits<E::bits> &c, const ScaleFmt &sf, float (&acc)[32],
                                          bool (&poisoned)[32 / B])
{
    constexpr int W = E::bits, NB = 32 / B;
    constexpr bool kHw = HW && E::hw_dec != HW_NONE;
    // the chunk is one block of a hardware 6-bit format: BF6 = E3M2; FP6 = E2M3, of which E2M2
    // is the half with an even mantissa (same bias, same largest exponent: 6-bit code = 5-bit
    // code << 1)
    constexpr bool kChunkBf6 = E::x == 3 && E::y == 2 && B == 32;
    constexpr bool kChunkFp6 = E::x == 2 && (E::y == 2 || E::y == 3) && B == 32;
    constexpr bool kChunk6 = kChunkBf6 || kChunkFp6;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
        const int sc = (int)((c.sw >> (8 * n)) & 0xFFu);
        const int e = sc - sf.sbias;
        poisoned[n] = poisoned[n] || (sf.has_nan && sc == 255);
        const int field = kChunk6 ? e + 127 : e - E::beta + E::hw_dec_bias + 127;
        const bool ok = field >= 0 && field <= 254;
        float d[B];
        if (kHw && kChunk6 && __builtin_amdgcn_ballot_w64(!ok) == 0) {
            // the lane holds one whole hardware block: a single instruction decodes the 32 codes
            uint32_t s6[6];
            if (W == 5) {
                const uint32_t in5[5] = {c.cw[0], c.cw[1], c.cw[2], c.cw[3 < W ? 3 : 0], c.cw[4 < W ? 4 : 0]};
                widen_5_to_6(in5, s6);
            } else {
#pragma unroll
                for (int k = 0; k < 6; ++k) s6[k] = c.cw[k < W ? k : 0];
            }
            const u32x6 src = {s6[0], s6[1], s6[2], s6[3], s6[4], s6[5]};
            // inline assembly with an early-clobber result: through the builtin the register
            // allocator let the result registers overlap the per-lane scale register
            f32x32 r;
            const float hs6 = __uint_as_float((uint32_t)field << 23);
            if (kChunkBf6)
                asm("v_cvt_scalef32_pk32_f32_bf6 %0, %1, %2" : "=&v"(r) : "v"(src), "v"(hs6));
            else
                asm("v_cvt_scalef32_pk32_f32_fp6 %0, %1, %2" : "=&v"(r) : "v"(src), "v"(hs6));
#pragma unroll
            for (int j = 0; j < B; ++j) d[j] = r[j < 32 ? j : 0];
        } else if (kHw && __builtin_amdgcn_ballot_w64(!ok) == 0) {
            const float hs = __uint_as_float((uint32_t)field << 23);
            // B codes of block n, eight at a time
#pragma unroll
            for (int g = 0; g < B / 8; ++g) {
                // the 8 codes occupy 8b bits starting at bit first*b (positions are constants once
                // n and g are unrolled)
                const int first = n * B + g * 8;
                const uint32_t lo = stream_bits_rt<W>(c.cw, first * W, 4 * W);
                const uint32_t hi = stream_bits_rt<W>(c.cw, first * W + 4 * W, 4 * W);
                const uint64_t v8 = (uint64_t)lo | ((uint64_t)hi << (4 * W));
                float d8[8];
                decode_unit_hw<E>(v8, hs, d8);
#pragma unroll
                for (int j = 0; j < 8; ++j) d[g * 8 + j] = d8[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < B; ++j) {
                const uint32_t cj = stream_bits_rt<W>(c.cw, (n * B + j) * W, W);
                const uint32_t bits = ((cj & E::magmask) << (23 - E::y)) | ((cj >> (E::x + E::y)) << 31);
                d[j] = ldexpf(__uint_as_float(bits), e + 127 - E::beta);
            }
        }
#pragma unroll
        for (int j = 0; j < B; ++j) acc[n * B + j] += d[j];
    }
}

// Blocks that some rank marked non-finite become NaN.
template <int B>
__device__ __forceinline__ void apply_poison(float (&acc)[32], const bool (&poisoned)[32 / B])
{
#pragma unroll
    for (int n = 0; n < 32 / B; ++n)
        if (poisoned[n]) {
#pragma unroll
            for (int j = 0; j < B; ++j) acc[n * B + j] = __uint_as_float(0x7FC00000u);
        }
}

// The own rank's raw bfloat16 values of a wave tile: the lane's 32 values are 64 contiguous
// bytes; the wave loads its 4 KiB as contiguous 16-byte pieces (load_raw_pieces) and hands each
// lane its four through the wave's LDS tile (take_raw_chunk), instead of four loads per lane that
// each touch 64 different lines.
template <bool NTL>
__device__ __forceinline__ void load_raw_pieces(u32x4 (&pv)[4], const void *own_x, size_t wave_chunk0,
                                                int lane, size_t units)
{
    const u32x4 *src = (const u32x4 *)own_x + wave_chunk0 * 4;
    // a unit's 8 bfloat16 values are one piece
    const size_t own_pieces = wave_chunk0 * 4 < units ? units - wave_chunk0 * 4 : 0;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int g = k * 64 + lane;             // piece index within the wave's 4 KiB
        pv[k] = (size_t)g < own_pieces ? ld<NTL>(src + g) : u32x4{0u, 0u, 0u, 0u};
    }
}

__device__ __forceinline__ void take_raw_chunk(u32x4 *t, const u32x4 (&pv)[4], u32x4 (&own)[4], int lane)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int g = k * 64 + lane;
        const int l = g >> 2, c = g & 3;         // owner lane and its piece number
        t[l * 4 + ((c + l) & 3)] = pv[k];
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int c = 0; c < 4; ++c) own[c] = t[lane * 4 + ((c + lane) & 3)];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// The same for a full wave tile with loads that write LDS directly: the 256 pieces are requested
// here into `traw` (4 KiB); once the wave's vector-memory counter has reached zero, lane l finds
// its four pieces at traw[4 l .. 4 l + 3].
template <bool NTL>
__device__ __forceinline__ void request_raw_to_lds(u32x4 *traw, const void *own_x, size_t wave_chunk0, int lane)
{
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    const u32x4 *src = (const u32x4 *)own_x + wave_chunk0 * 4;
#pragma unroll
    for (int k = 0; k < 4; ++k)
        __builtin_amdgcn_global_load_lds((gptr)(src + k * 64 + lane), (lptr)(traw + k * 64), 16, 0, NTL ? 2 : 0);
}

// Writes the wave tile's sums.  Exchange through LDS: lane l owns output pieces l*OC .. l*OC+OC-1
// of the wave's tile; piece c is written to slot (c + l) % OC of the lane's row so that both the
// row-wise writes and the piece-wise reads spread over all banks.  The wave then writes its
// output as contiguous 1 KiB store instructions.
template <bool OUT_BF16, bool NTS, bool FULL = false>
__device__ __forceinline__ void store_sums(u32x4 *t, const float (&acc)[32], void *outp, size_t wave_chunk0,
                                           int lane, size_t units)
{
    constexpr int OC = OUT_BF16 ? 4 : 8;         // 16-byte output pieces per lane
#pragma unroll
    for (int c = 0; c < OC; ++c) {
        u32x4 v;
        if (OUT_BF16) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = f32x2_to_bf16x2_rne(acc[8 * c + 2 * j], acc[8 * c + 2 * j + 1]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = __float_as_uint(acc[4 * c + j]);
        }
        t[lane * OC + ((c + lane) & (OC - 1))] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    u32x4 *out = (u32x4 *)outp + wave_chunk0 * OC;
    // a unit's 8 sums are OC / 4 pieces; the tensor's last chunk may hold fewer than 4 units
    const size_t pieces_left = wave_chunk0 * 4 < units ? (units - wave_chunk0 * 4) * (OC / 4) : 0;
#pragma unroll
    for (int r = 0; r < OC; ++r) {
        const int g = r * 64 + lane;             // piece index within the tile
        const int l = g / OC, c = g % OC;
        const u32x4 v = t[l * OC + ((c + l) & (OC - 1))];
        if (FULL || (size_t)g < pieces_left) st<NTS>(out + g, v);
    }
}

// Fused form: quantizes the lane's 32 sums again (same rule as the quantizer applied to binary32
// input) and stores codes and scales.  The lane holds whole blocks, so block maximum, scale and
// codes need no other lane.  Every lane of the wave must call this (narrow scales are gathered
// across the wave).
template <class E, int B, bool NTS, bool HW, bool FULL = false>
__device__ __forceinline__ void requantize_sums(const float (&acc)[32], void *codes_out, void *scales_out,
                                                size_t wave_chunk0, int lane, size_t nchunks,
                                                const ScaleFmt &sf)
{
    constexpr int W = E::bits, NB = 32 / B;
    constexpr bool kHw = HW && E::hw != HW_NONE;
    constexpr bool kChunkBf6 = E::x == 3 && E::y == 2 && B == 32;
    const bool valid = FULL || wave_chunk0 + (size_t)lane < nchunks;
    uint32_t cw[W];
#pragma unroll
    for (int k = 0; k < W; ++k) cw[k] = 0u;
    uint32_t sbytes = 0;
#pragma unroll
    for (int n = 0; n < NB; ++n) {
        uint32_t m = 0;
#pragma unroll
        for (int j = 0; j < B; ++j) m = max(m, __float_as_uint(acc[n * B + j]) & 0x7FFFFFFFu);
        const int expfield = (int)(m >> 23);
        int sc = 0;
        if (kHw && kChunkBf6) {
            // one instruction rounds the lane's 32 sums to BF6 = E3M2 (same scale rule)
            const int unclamped = expfield - 127 - E::emax + sf.sbias;
            const bool finite = expfield != 255;
            sc = finite ? min(max(unclamped, 0), sf.smax) : sf.nonfinite;
            const int fld = sc - sf.sbias + 127;
            if (__builtin_amdgcn_ballot_w64(finite && (fld < 0 || fld > 254)) == 0) {
                // the instruction interleaves its two sources: result code 2j comes from the
                // first operand's element j, code 2j+1 from the second operand's
                f32x16 even, odd;
#pragma unroll
                for (int j = 0; j < 16; ++j) {
                    even[j] = acc[2 * j];
                    odd[j] = acc[2 * j + 1];
                }
                // Issued as inline assembly with an early-clobber result: through the builtin the
                // register allocator let the six result registers overlap the per-lane scale
                // register, and every code after the first two came out wrong.
                u32x6 q;
                const float hs = __uint_as_float((uint32_t)max(fld, 0) << 23);
                asm("v_cvt_scalef32_2xpk16_bf6_f32 %0, %1, %2, %3"
                    : "=&v"(q)
                    : "v"(even), "v"(odd), "v"(hs));
#pragma unroll
                for (int k = 0; k < W; ++k) cw[k] = finite ? q[k < 6 ? k : 0] : 0u;
                sbytes |= (uint32_t)sc << (8 * n);
                continue;
            }
        }
#pragma unroll
        for (int g = 0; g < B / 8; ++g) {
            const int first = n * B + g * 8;
            u32x4 w2[2];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                w2[0][j] = __float_as_uint(acc[first + j]);
                w2[1][j] = __float_as_uint(acc[first + 4 + j]);
            }
            const uint64_t packed = encode_unit<E, true, HW>(w2, expfield, sf, &sc);
            // 8b bits at bit first*b of the chunk's stream (constant positions)
            const int pos = first * W;
            cw[pos >> 5] |= (uint32_t)(packed << (pos & 31));
            if ((pos & 31) + 8 * W > 32) {
                const uint64_t rest = packed >> (32 - (pos & 31));
                cw[((pos >> 5) + 1) < W ? (pos >> 5) + 1 : 0] |= (uint32_t)rest;
                if ((pos & 31) + 8 * W > 64)
                    cw[((pos >> 5) + 2) < W ? (pos >> 5) + 2 : 0] |= (uint32_t)(rest >> 32);
            }
        }
        sbytes |= (uint32_t)sc << (8 * n);
    }
    if (valid) {
        uint32_t *cp = (uint32_t *)codes_out + wave_chunk0 * W + lane * W;
        if (W == 4) {
            st<NTS>((u32x4 *)cp, u32x4{cw[0], cw[1], cw[2], cw[3 < W ? 3 : 0]});
        } else if (W == 6) {
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int k = 0; k < 3; ++k)
                st<NTS>((u32x2 *)cp + k, u32x2{cw[(2 * k) < W ? 2 * k : 0], cw[(2 * k + 1) < W ? 2 * k + 1 : 0]});
        } else {
#pragma unroll
            for (int k = 0; k < W; ++k) st<NTS>(cp + k, cw[k]);
        }
        if (sf.sbits == 8) {
            uint8_t *sp = (uint8_t *)scales_out + wave_chunk0 * NB + lane * NB;
            if (NB == 1) *sp = (uint8_t)sbytes;
            else if (NB == 2) *(uint16_t *)sp = (uint16_t)sbytes;
            else *(uint32_t *)sp = sbytes;
        }
    }
    if (sf.sbits < 8 && wave_chunk0 < nchunks) {
        // packed scale stream: each lane contributes NB fields of s bits = one wider field
        uint32_t field = 0;
#pragma unroll
        for (int n = 0; n < NB; ++n) field |= ((sbytes >> (8 * n)) & 0xFFu) << (n * sf.sbits);
        const size_t left = nchunks - wave_chunk0;
        uint8_t *run = (uint8_t *)scales_out + ((wave_chunk0 * NB * (size_t)sf.sbits) >> 3);
        with_scale_width(sf.sbits, [&](auto w) {
            store_packed_fields<1, NB * decltype(w)::value>(run, valid ? field : 0u, (int)(left < 64 ? left : 64));
        });
    }
}

// Fetches the code dwords of RC ranks for a full wave tile (64 valid chunks) through LDS: a rank's
// 64 chunks are 16*W pieces of 16 bytes, piece p requested by lane p % 64 with a load that writes
// LDS directly (no registers in between), so every load instruction covers whole cache lines (a
// lane's own W dwords are 4*W bytes apart, and loading them directly touches each line with
// several instructions).  The pieces of RC ranks are requested here into the wave's LDS area
// `t` (RC * 16 * W pieces); once the wave has waited for its vector-memory counter to reach
// zero, read_codes_from_lds hands each lane its W dwords.  Rank i is fetched when `on[i]`.
template <int W, int RC, bool NTL>
__device__ __forceinline__ void request_codes_to_lds(u32x4 *t, const void *(&codes)[RC], const bool (&on)[RC],
                                                     size_t wave_chunk0, int lane)
{
    constexpr int NP = 16 * W;
    constexpr int K = (NP + 63) / 64;
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
#pragma unroll
    for (int i = 0; i < RC; ++i) {
        const u32x4 *src = (const u32x4 *)((const uint32_t *)codes[i] + wave_chunk0 * W);
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int p = k * 64 + lane;
            // lane l's 16 bytes land at the given LDS address + 16 * l
            if (on[i] && p < NP)
                __builtin_amdgcn_global_load_lds((gptr)(src + p), (lptr)(t + i * NP + k * 64), 16, 0, NTL ? 2 : 0);
        }
    }
}

// Rank slot i of the area filled by request_codes_to_lds: the lane's W dwords.
template <int W>
__device__ __forceinline__ void read_codes_from_lds(uint32_t (&cw)[W], const u32x4 *t, int i, int lane)
{
    constexpr int NP = 16 * W;
    const uint32_t *tw = (const uint32_t *)t + i * NP * 4 + lane * W;
    if (W % 2 == 0) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int k = 0; k < W / 2; ++k) {
            const u32x2 v = *(const u32x2 *)(tw + 2 * k);
            cw[(2 * k) < W ? 2 * k : 0] = v.x;
            cw[(2 * k + 1) < W ? 2 * k + 1 : 0] = v.y;
        }
    } else {
#pragma unroll
        for (int k = 0; k < W; ++k) cw[k] = tw[k];
    }
}

// One wave tile: decode and add the tp ranks' chunks, then write (or re-quantize) the sums.
//
// FAST = the common case, compiled without anything it does not need: the tile is 64 whole chunks
// (every tile but a tensor's last is), tp <= kFastRanks so that the rank loop unrolls over fixed
// indices (the ranks' pointers then arrive with the other kernel arguments instead of one
// dependent scalar load per rank), and the scale format is fixed by S8 (true: one byte per block;
// false: a narrower bit stream).  The other instance (FAST = false) takes whatever is left — a
// partial last tile, the 1 to 3 unit chunk that ends a tensor whose size is not a multiple of 32,
// more ranks — with each lane loading its own dwords under bounds checks, two ranks at a time.
constexpr int kFastRanks = 8;

template <class E, int B, bool OUT_BF16, int RC, bool NTL, bool NTS, bool HW, bool FUSED, bool OWN, bool VIA_LDS,
          bool FAST, bool S8>
__device__ __forceinline__ void reduce_wave_tile(const ReduceArgs &a, u32x4 *t, int raw_offset, size_t wave_chunk0,
                                                 int lane)
{
    constexpr int NB = 32 / B;                   // blocks (scales) per chunk
    constexpr int W = E::bits;                   // dwords of codes per chunk
    constexpr bool kDma = FAST && VIA_LDS;       // codes through LDS (full tiles only)
    constexpr bool kCoopScales = FAST && !S8;    // narrow scales of a full tile: one load per rank
    const size_t nchunks = (a.units + 3) / 4;    // the last one may hold only 1 to 3 units
    const bool valid = FAST || wave_chunk0 + (size_t)lane < nchunks;
    // units in this lane's chunk if it is the tensor's last, partial one, else 0
    const int tail_units = (!FAST && wave_chunk0 + (size_t)lane == a.units / 4) ? (int)(a.units & 3) : 0;
    const ScaleFmt sf = (FAST && S8) ? ScaleFmt{8, 127, 254, 255, 1} : a.sf;

    float acc[32];
#pragma unroll
    for (int j = 0; j < 32; ++j) acc[j] = kFoldStart;
    bool poisoned[NB];
#pragma unroll
    for (int n = 0; n < NB; ++n) poisoned[n] = false;

    // OWN: the fast instance has the raw pieces written straight into their own LDS area (behind
    // the staging / exchange area) and reads them when the own rank's turn comes; the general one
    // takes them through registers up front
    constexpr bool kRawDma = OWN && FAST;
    u32x4 *traw = t + raw_offset;
    u32x4 own[4];
    if constexpr (OWN) {
        if (kRawDma) {
            request_raw_to_lds<NTL>(traw, a.own_x, wave_chunk0, lane);
        } else {
            u32x4 pv[4];
            load_raw_pieces<NTL>(pv, a.own_x, wave_chunk0, lane, a.units);
            take_raw_chunk(t, pv, own, lane);
        }
    }

    // FAST: all rank pointers are fetched from the argument block up front, in two wide scalar
    // loads, instead of one pair per rank right before its use
    const void *cp_all[FAST ? kFastRanks : 1], *sp_all[FAST ? kFastRanks : 1];
    if (FAST) {
#pragma unroll
        for (int r = 0; r < kFastRanks; ++r) {
            cp_all[FAST ? r : 0] = a.codes[r];
            sp_all[FAST ? r : 0] = a.scales[r];
        }
    }

    // ranks r0 .. r0 + RC - 1
    auto group = [&](int r0) {
        ChunkBits<W> g[RC];
        bool on[RC];
        const void *cptr[RC];
#pragma unroll
        for (int i = 0; i < RC; ++i) {
            const int r = r0 + i;
            const int rr = FAST ? r : min(r, a.tp - 1);
            on[i] = r < a.tp && !(OWN && r == a.own_rank);
            cptr[i] = FAST ? cp_all[FAST ? rr : 0] : a.codes[rr];
            const void *sptr = FAST ? sp_all[FAST ? rr : 0] : a.scales[rr];
            // with codes fetched through LDS this loads the scales only
            load_chunk<E, B, NTL, kDma, kCoopScales>(g[i], cptr[i], sptr, wave_chunk0, lane, valid && on[i], sf,
                                                        a.units, FAST, tail_units);
        }
        if (kDma) {
            request_codes_to_lds<W, RC, NTL>(t, cptr, on, wave_chunk0, lane);
            __builtin_amdgcn_s_waitcnt(0);       // every counter at zero: the pieces are in LDS
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        }
#pragma unroll
        for (int i = 0; i < RC; ++i) {
            if (OWN && r0 + i == a.own_rank) {
                if (kRawDma) {
                    if (!kDma) {                 // no group has waited for the counters yet
                        __builtin_amdgcn_s_waitcnt(0);
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                    }
#pragma unroll
                    for (int k = 0; k < 4; ++k) own[k] = traw[lane * 4 + k];
                }
#pragma unroll
                for (int k = 0; k < 4; ++k) add_raw_bf16(own[k], acc + 8 * k);
            } else if (r0 + i < a.tp) {
                // each rank's dwords are fetched from LDS only when its turn comes
                if (kDma) read_codes_from_lds<W>(g[i].cw, t, i, lane);
                if (kCoopScales) g[i].sw = spread_scale_fields<NB>(g[i].sw, lane, sf.sbits);
                add_chunk<E, B, HW>(g[i], sf, acc, poisoned);
            }
        }
        if (kDma) {
            // the area is free again once every lane has read its dwords
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    };
    if (FAST) {
#pragma unroll
        for (int r0 = 0; r0 < kFastRanks; r0 += RC)
            if (r0 < a.tp) group(r0);
    } else {
        for (int r0 = 0; r0 < a.tp; r0 += RC) group(r0);
    }
    apply_poison<B>(acc, poisoned);
    if (FUSED)
        requantize_sums<E, B, NTS, HW, FAST>(acc, a.codes_out, a.scales_out, wave_chunk0, lane, a.units / 4, sf);
    else
        store_sums<OUT_BF16, NTS, FAST>(t, acc, a.out, wave_chunk0, lane, a.units);
}

// The kernel: one wave per wave tile, no workgroup barrier.
//
// RC: ranks whose loads are issued together (a divisor of kFastRanks).  FUSED: instead of storing
// the sums, quantize them again in the lane that holds them and store codes and scales;
// bit-identical to running the unfused kernels one after the other.  OWN: rank a.own_rank
// contributes its uncompressed bf16 partial.  VIA_LDS: the codes of a full tile are fetched
// through LDS (request_codes_to_lds) instead of by each lane loading its own dwords.  WG: threads
// per workgroup (a multiple of 64).
template <class E, int B, bool OUT_BF16, int RC, bool NTL, bool NTS, bool HW, bool FUSED = false,
          bool OWN = false, int WG = kThreads, bool VIA_LDS = false>
__global__ __launch_bounds__(WG) void dequant_reduce_tile_kernel(ReduceArgs a)
{
    static_assert(!(FUSED && OWN), "the fused form has no own-raw variant");
    static_assert(kFastRanks % RC == 0, "RC must divide kFastRanks");
    constexpr int W = E::bits;
    constexpr int OC = OUT_BF16 ? 4 : 8;         // 16-byte output pieces per lane
    // LDS per wave, in 16-byte pieces: the output exchange, the staging of code pieces and the
    // own rank's raw pieces use the same area one after the other
    constexpr int kOutPieces = FUSED ? 0 : 64 * OC;
    constexpr int kStagePieces = VIA_LDS ? RC * 16 * W : 0;
    constexpr int kMainPieces = kOutPieces > kStagePieces ? kOutPieces : kStagePieces;
    // OWN: the raw pieces get 256 more behind it (the general instance, which passes them
    // through the main area, needs at least as many there)
    constexpr int kPieces = OWN ? (kMainPieces > 256 ? kMainPieces : 256) + 256 : kMainPieces;
    constexpr int kRawOffset = OWN ? kPieces - 256 : 0;
    __shared__ u32x4 tile[WG / 64][kPieces > 0 ? kPieces : 1];

    const int lane = (int)(threadIdx.x & 63);
    // the wave index is the same in every lane: telling the compiler so keeps wave_chunk0 and
    // every base address derived from it in scalar registers, and the per-lane part of an
    // address a 32-bit offset
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const size_t wave_chunk0 = ((size_t)blockIdx.x * (WG / 64) + (size_t)wave) * 64;
    if (wave_chunk0 * 4 >= a.units) return;      // the whole wave
    u32x4 *t = tile[kPieces > 0 ? wave : 0];
    const bool fast = wave_chunk0 + 64 <= a.units / 4 && a.tp <= kFastRanks;
    if (fast && a.sf.sbits == 8)
        reduce_wave_tile<E, B, OUT_BF16, RC, NTL, NTS, HW, FUSED, OWN, VIA_LDS, true, true>(a, t, kRawOffset, wave_chunk0, lane);
    else if (fast)
        reduce_wave_tile<E, B, OUT_BF16, RC, NTL, NTS, HW, FUSED, OWN, VIA_LDS, true, false>(a, t, kRawOffset, wave_chunk0, lane);
    else
        reduce_wave_tile<E, B, OUT_BF16, (RC > 2 ? 2 : RC), NTL, NTS, HW, FUSED, OWN, false, false, false>(a, t, kRawOffset, wave_chunk0,
                                                                                               lane);
}

// ---------------------------------------------------------------------------------------------
// Half-chunk form of the reduce kernel for E2M1 codes (any block size, any scale width), at most
// kFastRanks ranks and a tensor of whole wave tiles.  A lane owns 16 consecutive elements (half a
// chunk), a wave 1024, a workgroup of 512 threads 8192: the same bytes per workgroup as the tile
// form, in waves half as large and twice as many.  A launch of this form gets going and drains
// faster: 9 % less time at 1024 x 8192 elements and 8 ranks, 4 % at 4096 x 8192, 1 % at
// 6144 x 8192; beyond that the two forms move the same bytes per second (and this one loses
// 2-4 % when the ranks' buffers are 34 or 68 MiB apart), so the host uses it up to
// kHalfFormMaxUnits.  With few ranks the launch is mostly its float32 output and the tile form's
// larger waves do better (2 ranks: 1-15 % at every size; 4 ranks: 4-30 % below 4096 x 8192,
// 2-3 % worse above), so it is used from kHalfFormMinRanks ranks on.  The lane's codes are 8 contiguous bytes per rank, one 64-bit load; every
// scale code gives an exponent field the conversion accepts, so there is one decode path; the 16
// sums leave through the wave's LDS area as contiguous 128-bit stores, or (fused form) are
// quantized again by the lane, which shares a block of 32 with its neighbour.  For the 6-bit
// hardware formats the same shape decodes 16 codes with the 32-code conversion; with the codes
// fetched through LDS it gains 2 % (E3M2), so they stay on the tile form.
constexpr int kHalfThreads = 512;
constexpr size_t kHalfFormMaxUnits = (size_t)6144 * 8192 / 8;
constexpr int kHalfFormMinRanks = 6;

template <class E>
constexpr bool kHalfFormOk = E::hw == HW_FP4;

// TP: the number of ranks (kHalfFormMinRanks..kFastRanks), a compile-time constant so that the
// rank pointers come in one wide scalar load and all loads are issued before the first wait.
template <class E, int B, bool OUT_BF16, bool OWN, bool FUSED, bool NTL, bool NTS, int TP, bool S8>
__device__ __forceinline__ void reduce_wave_half(const ReduceArgs &a, u32x4 *t, u32x4 *traw, size_t half0, int lane)
{
    static_assert(kHalfFormOk<E>, "format not covered by the half-chunk form");
    constexpr int NBH = B >= 16 ? 1 : 16 / B;    // blocks whose scale the lane holds (1 or 2)
    constexpr int ND = 2 / NBH;                  // dwords (8 codes each) under one scale
    constexpr int OC = OUT_BF16 ? 2 : 4;         // 16-byte output pieces per lane
    const int sbits = S8 ? 8 : a.sf.sbits;
    const int sbias = S8 ? 127 : a.sf.sbias;

    // OWN: the wave's 2 KiB of the own rank's raw values are written straight into their LDS area
    // as 128 contiguous pieces; lane l finds its two at traw[2 l], traw[2 l + 1]
    if constexpr (OWN) {
        typedef const void __attribute__((address_space(1))) *gptr;
        typedef void __attribute__((address_space(3))) *lptr;
        const u32x4 *src = (const u32x4 *)a.own_x + half0 * 2;
#pragma unroll
        for (int k = 0; k < 2; ++k)
            __builtin_amdgcn_global_load_lds((gptr)(src + k * 64 + lane), (lptr)(traw + k * 64), 16, 0, NTL ? 2 : 0);
    }

    u32x2 cw[TP];
    uint32_t sw[TP];
#pragma unroll
    for (int r = 0; r < TP; ++r) {
        if (OWN && r == a.own_rank) continue;    // that rank's codes are not read
        cw[r] = ld<NTL>((const u32x2 *)a.codes[r] + half0 + (size_t)lane);
        const uint8_t *sp = (const uint8_t *)a.scales[r];
        if (!S8) {
            // narrow scales: the wave's 1024 / B fields are a dword-aligned run of the bit
            // stream, fetched one dword per lane and spread below
            const int ndw = (1024 / B) * sbits / 32;
            const uint32_t *run = (const uint32_t *)(sp + ((half0 * 16 / B * (size_t)sbits) >> 3));
            sw[r] = lane < ndw ? ld<NTL>(run + lane) : 0u;
        } else if (B == 32) {                     // the block's byte, shared with the other half
            sw[r] = ld<NTL>(sp + half0 / 2 + (size_t)(lane >> 1));
        } else if (B == 16) {
            sw[r] = ld<NTL>(sp + half0 + (size_t)lane);
        } else {
            sw[r] = ld<NTL>((const uint16_t *)sp + half0 + (size_t)lane);
        }
    }

    float acc[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) acc[j] = kFoldStart;
    bool poisoned[NBH];
#pragma unroll
    for (int n = 0; n < NBH; ++n) poisoned[n] = false;

    if constexpr (OWN) {
        __builtin_amdgcn_s_waitcnt(0);           // every counter at zero: the raw pieces are in LDS
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
#pragma unroll
    for (int r = 0; r < TP; ++r) {
        if (OWN && r == a.own_rank) {
            add_raw_bf16(traw[lane * 2], acc);
            add_raw_bf16(traw[lane * 2 + 1], acc + 8);
            continue;
        }
        // the lane's first block within the wave: lanes 2k and 2k + 1 share a block of 32
        if (!S8) sw[r] = spread_scale_fields_at<NBH>(sw[r], B == 32 ? lane >> 1 : lane * NBH, sbits);
#pragma unroll
        for (int n = 0; n < NBH; ++n) {
            // a scale byte is the exponent field the conversion takes (code 255 marks a
            // non-finite block: its sums are replaced below); a narrow code is re-biased to one
            const uint32_t sc = (sw[r] >> (8 * n)) & 0xFFu;
            poisoned[n] = poisoned[n] || (S8 && sc == 255u);
            const float hs = __uint_as_float((S8 ? min(sc, 254u) : sc + (uint32_t)(127 - sbias)) << 23);
#pragma unroll
            for (int h = 0; h < ND; ++h) {
                const uint32_t v = cw[r][n * ND + h];
                float *d = acc + 8 * (n * ND + h);
                const f32x2 r0 = cvt_fp4_pair<0>(v, hs), r1 = cvt_fp4_pair<1>(v, hs);
                const f32x2 r2 = cvt_fp4_pair<2>(v, hs), r3 = cvt_fp4_pair<3>(v, hs);
                d[0] += r0.x; d[1] += r0.y; d[2] += r1.x; d[3] += r1.y;
                d[4] += r2.x; d[5] += r2.y; d[6] += r3.x; d[7] += r3.y;
            }
        }
    }
#pragma unroll
    for (int n = 0; n < NBH; ++n)
        if (poisoned[n]) {
#pragma unroll
            for (int j = 0; j < 16 / NBH; ++j) acc[n * (16 / NBH) + j] = __uint_as_float(0x7FC00000u);
        }

    if constexpr (FUSED) {
        // quantize the sums again, with the quantizer's rule on binary32 input: a block of 32 is
        // shared with the neighbouring lane, smaller blocks are the lane's own
        const ScaleFmt sf = S8 ? ScaleFmt{8, 127, 254, 255, 1} : a.sf;
        u32x2 cq = {0u, 0u};
        uint32_t sq = 0;                         // the lane's NBH scale codes, sbits apart
#pragma unroll
        for (int n = 0; n < NBH; ++n) {
            uint32_t m = 0;
#pragma unroll
            for (int j = 0; j < 16 / NBH; ++j) m = max(m, __float_as_uint(acc[n * (16 / NBH) + j]) & 0x7FFFFFFFu);
            if (B == 32) m = max(m, dpp<quad_perm(1, 0, 3, 2)>(m));
            int sc = 0;
#pragma unroll
            for (int h = 0; h < ND; ++h) {
                const float *d = acc + 8 * (n * ND + h);
                const u32x4 w2[2] = {{__float_as_uint(d[0]), __float_as_uint(d[1]), __float_as_uint(d[2]), __float_as_uint(d[3])},
                                     {__float_as_uint(d[4]), __float_as_uint(d[5]), __float_as_uint(d[6]), __float_as_uint(d[7])}};
                cq[n * ND + h] = (uint32_t)encode_unit<E, true, true>(w2, (int)(m >> 23), sf, &sc);
            }
            sq |= (uint32_t)sc << (n * sbits);
        }
        st<NTS>((u32x2 *)a.codes_out + half0 + (size_t)lane, cq);
        uint8_t *sp = (uint8_t *)a.scales_out;
        if (!S8) {
            // the wave's 1024 / B fields are a whole number of bytes of the stream
            uint8_t *run = sp + ((half0 * 16 / B * (size_t)sbits) >> 3);
            with_scale_width(sbits, [&](auto w) {
                if (B == 32) store_packed_fields<2, decltype(w)::value>(run, sq, 32);
                else store_packed_fields<1, NBH * decltype(w)::value>(run, sq, 64);
            });
        } else if (B == 32) {
            if ((lane & 1) == 0) sp[half0 / 2 + (size_t)(lane >> 1)] = (uint8_t)sq;
        } else if (B == 16) {
            sp[half0 + (size_t)lane] = (uint8_t)sq;
        } else {
            ((uint16_t *)sp)[half0 + (size_t)lane] = (uint16_t)sq;
        }
        return;
    }

    // exchange through LDS as in store_sums: piece c of lane l sits at slot (c + l) % OC of row l
#pragma unroll
    for (int c = 0; c < OC; ++c) {
        u32x4 v;
        if (OUT_BF16) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[j] = f32x2_to_bf16x2_rne(acc[8 * c + 2 * j], acc[8 * c + 2 * j + 1]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = __float_as_uint(acc[4 * c + j]);
        }
        t[lane * OC + ((c + lane) & (OC - 1))] = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    u32x4 *out = (u32x4 *)a.out + half0 * OC;
#pragma unroll
    for (int k = 0; k < OC; ++k) {
        const int g = k * 64 + lane;             // piece index within the wave's output
        const int l = g / OC, c = g % OC;
        st<NTS>(out + g, t[l * OC + ((c + l) & (OC - 1))]);
    }
}

template <class E, int B, bool OUT_BF16, bool OWN, bool FUSED, bool NTL, bool NTS>
__global__ __launch_bounds__(kHalfThreads) void dequant_reduce_half_kernel(ReduceArgs a)
{
    static_assert(!(FUSED && OWN), "the fused form has no own-raw variant");
    constexpr int OC = FUSED ? 0 : OUT_BF16 ? 2 : 4;
    // per wave: the output exchange area, and behind it the own rank's raw pieces
    constexpr int kPieces = 64 * OC + (OWN ? 128 : 0);
    __shared__ u32x4 tile[kHalfThreads / 64][kPieces > 0 ? kPieces : 1];
    const int lane = (int)(threadIdx.x & 63);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // first half-chunk of the wave; a half-chunk is two units
    const size_t half0 = ((size_t)blockIdx.x * (kHalfThreads / 64) + (size_t)wave) * 64;
    if (half0 * 2 >= a.units) return;            // the whole wave
    if (a.tp < kHalfFormMinRanks || a.tp > kFastRanks) return;   // the host never launches this
    u32x4 *t = tile[kPieces > 0 ? wave : 0];
    // the rank count and the scale width become compile-time constants of the body
    auto with_tp = [&](auto s8) {
        constexpr bool S8 = decltype(s8)::value;
        switch (a.tp) {
        case 6: reduce_wave_half<E, B, OUT_BF16, OWN, FUSED, NTL, NTS, 6, S8>(a, t, t + 64 * OC, half0, lane); break;
        case 7: reduce_wave_half<E, B, OUT_BF16, OWN, FUSED, NTL, NTS, 7, S8>(a, t, t + 64 * OC, half0, lane); break;
        default: reduce_wave_half<E, B, OUT_BF16, OWN, FUSED, NTL, NTS, 8, S8>(a, t, t + 64 * OC, half0, lane); break;
        }
    };
    if (a.sf.sbits == 8) with_tp(std::true_type{});
    else with_tp(std::false_type{});
}

}  // namespace mxc
