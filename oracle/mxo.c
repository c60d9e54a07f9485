/*
 * mxo — plain CPU oracle for block (microscaling-style) communication compression.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute; it is
 * called from tests, from the smoke check and from the benchmark's CPU-baseline leg, and from
 * nowhere else.  It shares no code, header, table or constant with the HIP path.
 *
 * What it follows (paper sections, restated):
 *   - Method, "Communication Compression": every worker of a tensor-parallel group compresses
 *     the partial result of a row-wise linear layer with fine-grained block-wise quantization —
 *     a block of values is stored in a low-bit floating-point element format together with one
 *     shared power-of-two exponent — and decompresses before the reduction.
 *   - Method, parameter list: element formats FP5 (E3M1, E2M2, E1M3), FP4 (E2M1, E1M2),
 *     FP3 (E1M1) and INT3/4/5 (which the ablation table shows equal to the E1My formats);
 *     block sizes 8/16/32; scale formats E8M0 ... E4M0.
 *   - Profiling: the N decompressed partials are reduced with a plain sum.
 *   - Model Evaluation / Table 1 / Table 3 caption: effective bits = element bits +
 *     scale bits / block size.
 *
 * The paper gives no formula for the shared exponent, the rounding or the byte layout; the
 * readings used here are:
 *   element ExMy : sign-magnitude, b = 1+x+y bits, code = sign<<(x+y) | exp<<y | mant,
 *                  bias beta = 2^(x-1)-1, no Inf/NaN codes, exp==0 is subnormal
 *                  2^(1-beta) * mant/2^y, otherwise 2^(exp-beta) * (1 + mant/2^y);
 *                  emax = 2^x - 1 - beta, maxval = 2^emax * (2 - 2^-y).
 *   scale EsM0   : code = e + sbias, sbias = 2^(s-1)-1, value 2^e.  s = 8: codes 0..254 and
 *                  255 marks a block that held an Inf/NaN.  s < 8: codes 0..2^s-1, no marker.
 *   shared exp   : e = clamp(floor(log2(max|v|)) - emax) to the scale's range.
 *   element      : nearest ExMy magnitude to |v| * 2^-e, ties to the even code, saturating at
 *                  maxval; the sign bit is the input's sign bit, always.
 *   non-finite   : a block with any Inf/NaN stores all-zero element codes and the marker scale
 *                  (s = 8) or the largest scale code (s < 8).
 *   packing      : element j of a row occupies bits [j*b, (j+1)*b) of the row's little-endian
 *                  bit stream.  Scales: s = 8 one byte per block, row-major; s < 8 a bit stream
 *                  over all blocks of the tensor, block k at bits [k*s, (k+1)*s), LSB first,
 *                  the last byte padded with zeros (mxo_pack_scales).
 *   reduction    : out = (((d0 + d1) + d2) + ...), IEEE binary32 adds in rank order, d_r the
 *                  exactly decoded value (a scale byte of 255 decodes the block to NaN).
 *
 * All value arithmetic is done on doubles with frexp/ldexp/nearbyint: every quantity that
 * appears (inputs with <= 24 significant bits times a power of two) is exact in a double, so
 * there is no rounding here other than the one the method itself prescribes.
 *
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fopenmp -shared -fPIC mxo.c -o libmxo.so -lm
 */
#include <fenv.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t ebits;      /* x: exponent bits of an element, 1..3 */
    int32_t mbits;      /* y: mantissa bits of an element, 1..4 */
    int32_t block;      /* B: elements per shared scale */
    int32_t scale_bits; /* s: 4..8 */
} mxo_format;

enum { MXO_OK = 0, MXO_ERR_FORMAT = -2, MXO_ERR_SHAPE = -3, MXO_ERR_TP = -5 };

/* ------------------------------------------------------------------ format facts ---------- */

static int fmt_bits(const mxo_format *f) { return 1 + f->ebits + f->mbits; }
static int fmt_beta(const mxo_format *f) { return (1 << (f->ebits - 1)) - 1; }
static int fmt_emax(const mxo_format *f) { return (1 << f->ebits) - 1 - fmt_beta(f); }
static double fmt_maxval(const mxo_format *f)
{
    return ldexp(2.0 - ldexp(1.0, -f->mbits), fmt_emax(f));
}
static int scale_bias(const mxo_format *f) { return (1 << (f->scale_bits - 1)) - 1; }
static int scale_maxcode(const mxo_format *f)
{
    return f->scale_bits == 8 ? 254 : (1 << f->scale_bits) - 1;
}

static int fmt_ok(const mxo_format *f)
{
    if (!f) return 0;
    if (f->ebits < 1 || f->ebits > 3) return 0;
    if (f->mbits < 1 || f->mbits > 4) return 0;
    if (fmt_bits(f) < 3 || fmt_bits(f) > 6) return 0;
    if (f->block != 8 && f->block != 16 && f->block != 32) return 0;
    if (f->scale_bits < 4 || f->scale_bits > 8) return 0;
    return 1;
}

int mxo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Effective bits per element and the sizes of the packed arrays (Model Evaluation; Table 1
 * column 3; Table 3 caption).  scale_bytes is ceil(blocks*s/8): whenever blocks*s is a multiple
 * of 8 the two arrays together are exactly effective_bits per element. */
int mxo_packed_sizes(const mxo_format *f, int64_t tokens, int64_t hidden,
                     uint64_t *code_bytes, uint64_t *scale_bytes, double *effective_bits)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    uint64_t blocks = (uint64_t)tokens * (uint64_t)(hidden / f->block);
    if (code_bytes) *code_bytes = (uint64_t)tokens * (uint64_t)hidden * (uint64_t)fmt_bits(f) / 8u;
    if (scale_bytes) *scale_bytes = (blocks * (uint64_t)f->scale_bits + 7u) / 8u;
    if (effective_bits) *effective_bits = fmt_bits(f) + (double)f->scale_bits / f->block;
    return MXO_OK;
}

/* One scale code per byte -> the array that travels: unchanged for s = 8, an s-bit stream for
 * s < 8 (block k at bits [k*s, (k+1)*s), LSB first, zero padding in the last byte). */
int mxo_pack_scales(const mxo_format *f, const uint8_t *scale_codes, int64_t nblocks, uint8_t *packed)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (nblocks < 0) return MXO_ERR_SHAPE;
    int s = f->scale_bits;
    if (s == 8) { memcpy(packed, scale_codes, (size_t)nblocks); return MXO_OK; }
    memset(packed, 0, (size_t)((nblocks * s + 7) / 8));
    for (int64_t k = 0; k < nblocks; ++k)
        for (int b = 0; b < s; ++b) {
            int64_t bit = k * s + b;
            if ((scale_codes[k] >> b) & 1u) packed[bit >> 3] |= (uint8_t)(1u << (bit & 7));
        }
    return MXO_OK;
}

int mxo_unpack_scales(const mxo_format *f, const uint8_t *packed, int64_t nblocks, uint8_t *scale_codes)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (nblocks < 0) return MXO_ERR_SHAPE;
    int s = f->scale_bits;
    if (s == 8) { memcpy(scale_codes, packed, (size_t)nblocks); return MXO_OK; }
    for (int64_t k = 0; k < nblocks; ++k) {
        unsigned c = 0;
        for (int b = 0; b < s; ++b) {
            int64_t bit = k * s + b;
            c |= (unsigned)((packed[bit >> 3] >> (bit & 7)) & 1u) << b;
        }
        scale_codes[k] = (uint8_t)c;
    }
    return MXO_OK;
}

/* Value of one element code (sign included), before the block scale is applied. */
double mxo_code_value(const mxo_format *f, unsigned code)
{
    int x = f->ebits, y = f->mbits, beta = fmt_beta(f);
    unsigned mant = code & ((1u << y) - 1u);
    unsigned expf = (code >> y) & ((1u << x) - 1u);
    unsigned sign = (code >> (x + y)) & 1u;
    double mag;
    if (expf == 0)
        mag = ldexp((double)mant, 1 - beta - y);
    else
        mag = ldexp(1.0 + ldexp((double)mant, -y), (int)expf - beta);
    return sign ? -mag : mag;
}

/* Value of a scale byte: 2^(code - sbias); NaN for the non-finite marker of an 8-bit scale. */
double mxo_scale_value(const mxo_format *f, unsigned code)
{
    if (f->scale_bits == 8 && code == 255u) return NAN;
    return ldexp(1.0, (int)code - scale_bias(f));
}

/* ------------------------------------------------------------------ input decoding -------- */

/* bfloat16 bit pattern -> its real value (sign, 8 exponent bits, 7 fraction bits). */
static double bf16_value(uint16_t h)
{
    int sign = h >> 15, ex = (h >> 7) & 0xFF, fr = h & 0x7F;
    double mag;
    if (ex == 0xFF)
        mag = fr ? NAN : INFINITY;
    else if (ex == 0)
        mag = ldexp((double)fr, -126 - 7);
    else
        mag = ldexp((double)(128 + fr), ex - 127 - 7);
    return sign ? -mag : mag;
}

/* ------------------------------------------------------------------ one block ------------- */

/* Magnitude code of the ExMy value nearest to p >= 0 (ties to even, saturating). */
static unsigned nearest_magnitude_code(const mxo_format *f, double p)
{
    int x = f->ebits, y = f->mbits, beta = fmt_beta(f);
    (void)x;
    if (p == 0.0) return 0u;

    int k;
    (void)frexp(p, &k);                 /* p = m * 2^k, m in [0.5, 1)  =>  floor(log2 p) = k-1 */
    int binade = k - 1;
    if (binade < 1 - beta) binade = 1 - beta;       /* subnormals share the lowest binade's step */
    double quantum = ldexp(1.0, binade - y);
    double q = nearbyint(p / quantum) * quantum;    /* p/quantum is exact; ties go to even */
    double maxval = fmt_maxval(f);
    if (q > maxval) q = maxval;

    /* encode q, which is now exactly an ExMy magnitude */
    double min_normal = ldexp(1.0, 1 - beta);
    if (q < min_normal) return (unsigned)(q / ldexp(1.0, 1 - beta - y));
    int kq;
    double mq = frexp(q, &kq);          /* q = mq * 2^kq, mq in [0.5,1) => q = (2mq) * 2^(kq-1) */
    unsigned expf = (unsigned)(kq - 1 + beta);
    unsigned mant = (unsigned)((2.0 * mq - 1.0) * (double)(1 << y));
    return (expf << y) | mant;
}

/* Quantize B values (already as doubles, exact).  codes[i] gets the b-bit code in the low bits
 * of one byte; *scale gets the scale byte. */
static void quantize_block(const mxo_format *f, const double *v, uint8_t *codes, uint8_t *scale)
{
    int B = f->block, x = f->ebits, y = f->mbits;
    int finite = 1;
    double m = 0.0;
    for (int i = 0; i < B; ++i) {
        if (!isfinite(v[i])) finite = 0;
        else if (fabs(v[i]) > m) m = fabs(v[i]);
    }
    if (!finite) {
        *scale = (uint8_t)(f->scale_bits == 8 ? 255 : scale_maxcode(f));
        memset(codes, 0, (size_t)B);
        return;
    }
    int sbias = scale_bias(f), smax = scale_maxcode(f);
    int sc;
    if (m == 0.0) {
        sc = 0;                                     /* floor(log2 0) = -inf: lowest scale */
    } else {
        int k;
        (void)frexp(m, &k);
        long e = (long)(k - 1) - fmt_emax(f);       /* shared exponent */
        long c = e + sbias;
        sc = c < 0 ? 0 : (c > smax ? smax : (int)c);
    }
    *scale = (uint8_t)sc;
    int e = sc - sbias;
    for (int i = 0; i < B; ++i) {
        double p = ldexp(fabs(v[i]), -e);           /* exact */
        unsigned mag = nearest_magnitude_code(f, p);
        unsigned sign = signbit(v[i]) ? 1u : 0u;
        codes[i] = (uint8_t)((sign << (x + y)) | mag);
    }
}

/* ------------------------------------------------------------------ tensors --------------- */

/* Quantize a bf16 [tokens x hidden] tensor, blocks along hidden.  Writes one code per byte
 * (codes_unpacked, tokens*hidden) and one scale byte per block (tokens*hidden/B). */
int mxo_quantize_bf16(const mxo_format *f, const uint16_t *x, int64_t tokens, int64_t hidden,
                      uint8_t *codes_unpacked, uint8_t *scales)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    fesetround(FE_TONEAREST);
    int B = f->block;
    int64_t nb = hidden / B;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t) {
        fesetround(FE_TONEAREST);
        double v[32];
        for (int64_t j = 0; j < nb; ++j) {
            const uint16_t *src = x + t * hidden + j * B;
            for (int i = 0; i < B; ++i) v[i] = bf16_value(src[i]);
            quantize_block(f, v, codes_unpacked + t * hidden + j * B, scales + t * nb + j);
        }
    }
    return MXO_OK;
}

/* Same for a binary32 input (the reduced tensor that is quantized again per chunk). */
int mxo_quantize_f32(const mxo_format *f, const float *x, int64_t tokens, int64_t hidden,
                     uint8_t *codes_unpacked, uint8_t *scales)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    fesetround(FE_TONEAREST);
    int B = f->block;
    int64_t nb = hidden / B;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t) {
        fesetround(FE_TONEAREST);
        double v[32];
        for (int64_t j = 0; j < nb; ++j) {
            const float *src = x + t * hidden + j * B;
            for (int i = 0; i < B; ++i) v[i] = (double)src[i];
            quantize_block(f, v, codes_unpacked + t * hidden + j * B, scales + t * nb + j);
        }
    }
    return MXO_OK;
}

/* One-code-per-byte -> packed bit stream (row-major, LSB first). */
int mxo_pack(const mxo_format *f, const uint8_t *codes_unpacked, int64_t tokens, int64_t hidden,
             uint8_t *packed)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    int b = fmt_bits(f);
    int64_t row_bytes = hidden * b / 8;
    memset(packed, 0, (size_t)(tokens * row_bytes));
    for (int64_t t = 0; t < tokens; ++t) {
        uint8_t *row = packed + t * row_bytes;
        for (int64_t j = 0; j < hidden; ++j) {
            unsigned c = codes_unpacked[t * hidden + j];
            for (int k = 0; k < b; ++k) {
                int64_t bit = j * b + k;
                if ((c >> k) & 1u) row[bit >> 3] |= (uint8_t)(1u << (bit & 7));
            }
        }
    }
    return MXO_OK;
}

/* Packed bit stream -> one code per byte. */
int mxo_unpack(const mxo_format *f, const uint8_t *packed, int64_t tokens, int64_t hidden,
               uint8_t *codes_unpacked)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    int b = fmt_bits(f);
    int64_t row_bytes = hidden * b / 8;
    for (int64_t t = 0; t < tokens; ++t) {
        const uint8_t *row = packed + t * row_bytes;
        for (int64_t j = 0; j < hidden; ++j) {
            unsigned c = 0;
            for (int k = 0; k < b; ++k) {
                int64_t bit = j * b + k;
                c |= (unsigned)((row[bit >> 3] >> (bit & 7)) & 1u) << k;
            }
            codes_unpacked[t * hidden + j] = (uint8_t)c;
        }
    }
    return MXO_OK;
}

/* Decode one rank: d[t,h] = value(code) * 2^(scale - sbias), as binary32 (exact). */
int mxo_dequantize(const mxo_format *f, const uint8_t *codes_unpacked, const uint8_t *scales,
                   int64_t tokens, int64_t hidden, float *out)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    int B = f->block;
    int64_t nb = hidden / B;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            double s = mxo_scale_value(f, scales[t * nb + h / B]);
            double d = mxo_code_value(f, codes_unpacked[t * hidden + h]) * s;
            out[t * hidden + h] = (float)d;
        }
    return MXO_OK;
}

/* Decode the tp ranks and add them in rank order with binary32 adds, starting from rank 0's
 * value (not from +0).  codes_unpacked[r] / scales[r] are rank r's arrays. */
int mxo_dequant_reduce(const mxo_format *f, int tp, const uint8_t *const *codes_unpacked,
                       const uint8_t *const *scales, int64_t tokens, int64_t hidden, float *out)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tp < 1 || tp > 32) return MXO_ERR_TP;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    int B = f->block;
    int64_t nb = hidden / B;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            volatile float acc = 0.0f;
            for (int r = 0; r < tp; ++r) {
                double s = mxo_scale_value(f, scales[r][t * nb + h / B]);
                float d = (float)(mxo_code_value(f, codes_unpacked[r][t * hidden + h]) * s);
                if (r == 0) acc = d;
                else { float a = acc; acc = a + d; }
            }
            out[t * hidden + h] = acc;
        }
    return MXO_OK;
}

/* The reduction as the Profiling section words it: a worker decompresses the partials of the
 * N-1 other workers and adds its own partial as it is.  Same left fold in rank order, but the
 * term of rank own_rank is the bfloat16 value own_x[t,h] (exact in binary32);
 * codes_unpacked[own_rank] and scales[own_rank] are not read. */
int mxo_dequant_reduce_own(const mxo_format *f, int tp, int own_rank, const uint16_t *own_x,
                           const uint8_t *const *codes_unpacked, const uint8_t *const *scales,
                           int64_t tokens, int64_t hidden, float *out)
{
    if (!fmt_ok(f)) return MXO_ERR_FORMAT;
    if (tp < 1 || tp > 32 || own_rank < 0 || own_rank >= tp) return MXO_ERR_TP;
    if (tokens < 0 || hidden < 0 || hidden % f->block) return MXO_ERR_SHAPE;
    int B = f->block;
    int64_t nb = hidden / B;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < tokens; ++t)
        for (int64_t h = 0; h < hidden; ++h) {
            volatile float acc = 0.0f;
            for (int r = 0; r < tp; ++r) {
                float d;
                if (r == own_rank) {
                    d = (float)bf16_value(own_x[t * hidden + h]);
                } else {
                    double s = mxo_scale_value(f, scales[r][t * nb + h / B]);
                    d = (float)(mxo_code_value(f, codes_unpacked[r][t * hidden + h]) * s);
                }
                if (r == 0) acc = d;
                else { float a = acc; acc = a + d; }
            }
            out[t * hidden + h] = acc;
        }
    return MXO_OK;
}

/* binary32 -> bfloat16 bit pattern, round to nearest even; NaN -> 0x7FC0. */
static uint16_t bf16_from_float(float v)
{
    if (isnan(v)) return 0x7FC0;
    uint16_t sign = signbit(v) ? 0x8000 : 0;
    double a = fabs((double)v);
    if (isinf(a)) return (uint16_t)(sign | 0x7F80);
    if (a == 0.0) return sign;
    int k;
    (void)frexp(a, &k);
    int binade = k - 1;
    if (binade < -126) binade = -126;
    double quantum = ldexp(1.0, binade - 7);
    double q = nearbyint(a / quantum) * quantum;
    if (q >= ldexp(1.0, 128)) return (uint16_t)(sign | 0x7F80);
    if (q < ldexp(1.0, -126)) return (uint16_t)(sign | (uint16_t)(q / ldexp(1.0, -133)));
    int kq;
    double mq = frexp(q, &kq);
    unsigned ex = (unsigned)(kq - 1 + 127);
    unsigned fr = (unsigned)((2.0 * mq - 1.0) * 128.0);
    return (uint16_t)(sign | (ex << 7) | fr);
}

/* Round a binary32 tensor to bfloat16 bit patterns (the optional 16-bit output of the
 * reduction). */
int mxo_round_to_bf16(const float *x, int64_t n, uint16_t *out)
{
    fesetround(FE_TONEAREST);
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_from_float(x[i]);
    return MXO_OK;
}

/* The uncompressed reduction the method is compared with (Profiling: without compression the
 * partials are reduced as they are): out = (((x_0 + x_1) + x_2) + ...), binary32 adds in rank
 * order of the bfloat16 partials. */
int mxo_sum_bf16(int tp, const uint16_t *const *x, int64_t n, float *out)
{
    if (tp < 1 || tp > 32) return MXO_ERR_TP;
    if (n < 0) return MXO_ERR_SHAPE;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        volatile float acc = (float)bf16_value(x[0][i]);
        for (int r = 1; r < tp; ++r) {
            float a = acc;
            acc = a + (float)bf16_value(x[r][i]);
        }
        out[i] = acc;
    }
    return MXO_OK;
}

/* Quality proxy for a compressed reduction: signal-to-quantization-noise ratio in dB of `test`
 * against the uncompressed result `ref`, 10 log10( sum ref^2 / sum (test - ref)^2 ), both sums
 * accumulated in doubles in index order.  It stands in for the perplexity increase the Model
 * Evaluation section reports, which needs models and data.  Equal tensors give +infinity. */
int mxo_sqnr_db(const float *ref, const float *test, int64_t n, double *out)
{
    if (n < 0) return MXO_ERR_SHAPE;
    double signal = 0.0, noise = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double r = (double)ref[i], d = (double)test[i] - r;
        signal += r * r;
        noise += d * d;
    }
    *out = noise > 0.0 ? 10.0 * log10(signal / noise) : INFINITY;
    return MXO_OK;
}
