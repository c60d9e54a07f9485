/*
 * mxc — block-quantized communication compression for tensor-parallel partial activations,
 *       MI355X (gfx950) library.  C ABI: plain pointers and sizes only.
 *
 * The operations are those of the paper's Method section ("Communication Compression") and
 * Profiling section: every worker of a tensor-parallel group of N workers compresses the
 * partial result of a row-wise linear layer with fine-grained block-wise quantization (a block
 * of values stored in a low-bit floating-point element format plus one shared power-of-two
 * exponent), and after the exchange the N partials are decompressed and summed.  Format
 * parameters are the ones the Method section lists: element data type, block size, scale data
 * type.  mxc_requantize_chunk is this library's extension for a reduce-scatter / all-gather
 * split of the exchange (quantize a 1/N row chunk of the reduced tensor again); the paper only
 * has the all-gather form.
 *
 * Common rules
 *   1. Tensors are row-major [tokens x hidden]; blocks are `block` consecutive elements of one
 *      row, so hidden % block == 0 is required.
 *   2. Element format ExMy: sign-magnitude, b = 1 + ebits + mbits bits, code =
 *      sign << (x+y) | exp << y | mant, exponent bias 2^(x-1)-1, no Inf/NaN codes, exp == 0 is
 *      subnormal.  Scale EsM0: per block the code e + (2^(s-1)-1), the block's values being
 *      code_value * 2^e.
 *   3. Shared exponent e = floor(log2(max|v|)) - emax clamped to the scale's range; elements are
 *      rounded to the nearest magnitude, ties to the even code, saturating at the largest
 *      magnitude; the sign bit is the input's sign bit.
 *   4. Non-finite input, 8-bit scales: a block containing an Inf or NaN stores all-zero codes
 *      and scale byte 255, and scale byte 255 decodes the whole block to NaN.  The NaN therefore
 *      reaches the reduced output on every worker.
 *   5. Non-finite input, scales narrower than 8 bits: there is NO marker.  A block containing an
 *      Inf or NaN stores all-zero codes and the largest scale code, and decodes to zeros: the
 *      non-finite value is LOST, silently, and the reduced output is finite.  With
 *      mxc_dequant_reduce_own the worker that owns the block adds its raw Inf/NaN and gets a
 *      non-finite sum while every other worker gets a finite one, so the replicas of the
 *      reduced tensor differ in that block.  Callers that may see non-finite activations and
 *      need them to propagate must use an 8-bit scale.
 *   6. Packed codes: element j of a row occupies bits [j*b, (j+1)*b) of the row's little-endian
 *      bit stream, rows back to back (hidden*b/8 bytes each).  Scales, s = 8: uint8 [tokens x
 *      hidden/block], row-major.  Scales, s < 8: a bit stream over all blocks of the tensor in
 *      the same order, block k at bits [k*s, (k+1)*s), LSB first, ceil(blocks*s/8) bytes, unused
 *      bits of the last byte zero.
 *   7. Every data pointer is a DEVICE pointer owned by the caller, valid until the stream has
 *      finished the call.  Arrays of pointers (`const void* const*`) are HOST arrays of device
 *      pointers; they are read during the call and need not outlive it.  The library cannot see
 *      buffer sizes: a buffer shorter than the shape implies is read or written past its end.
 *   8. `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Each call
 *      validates its arguments on the host, enqueues one kernel on that stream and returns
 *      without synchronising.  The library allocates nothing and keeps no state (other than the
 *      pair of events mxc_time_next_launch arms for one launch of the calling thread).
 *   9. Return value: MXC_OK or a negative mxc_status.  On error nothing has been enqueued.  A
 *      valid call on an empty tensor (tokens == 0) enqueues nothing and returns MXC_OK.
 *      MXC_ERR_HIP reports the launch call's own return value; the thread's HIP error state is
 *      neither read nor cleared.
 *  10. Alignment: bf16/f32 tensors and packed code arrays must be 16-byte aligned, scale arrays
 *      4-byte aligned (MXC_ERR_ALIGN otherwise).  A requantize chunk's rows start at multiples of
 *      tokens/tp rows, which keeps this alignment for every supported shape.
 */
#ifndef MXC_H
#define MXC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Method, parameter list: value data type (ExMy), block size, scale data type (EsM0). */
typedef struct {
    int32_t ebits;      /* x, 1..3 */
    int32_t mbits;      /* y, 1..4; 3 <= 1+x+y <= 6 */
    int32_t block;      /* 8, 16 or 32 */
    int32_t scale_bits; /* s, 4..8 */
} mxc_format;

typedef enum {
    MXC_OK = 0,
    MXC_ERR_NULL = -1,   /* a required pointer is NULL */
    MXC_ERR_FORMAT = -2, /* unsupported element / block / scale format */
    MXC_ERR_SHAPE = -3,  /* non-positive size, hidden % block, tokens % tp, size overflow */
    MXC_ERR_ALIGN = -4,  /* a device pointer is not aligned as stated above */
    MXC_ERR_TP = -5,     /* tp outside 1..32, chunk outside 0..tp-1, batch count outside 1..32 */
    MXC_ERR_HIP = -6,    /* the HIP runtime refused the launch */
    MXC_ERR_DTYPE = -7   /* unknown mxc_dtype */
} mxc_status;

typedef enum { MXC_F32 = 0, MXC_BF16 = 1 } mxc_dtype;

#define MXC_MAX_TP 32

/* Human-readable text for a status code; never NULL. */
const char *mxc_strerror(int status);

/* Library version string, e.g. "mxc 0.2 gfx950". */
const char *mxc_version(void);

/* Sizes of the packed arrays for one [tokens x hidden] tensor (host only, closed form):
 * code_bytes = tokens*hidden*b/8, scale_bytes = ceil(tokens*hidden/block * s / 8).  Either output
 * pointer may be NULL.  (Model Evaluation: effective bits = b + s/block; the two arrays together
 * are exactly that many bits per element whenever the scale stream fills its last byte.) */
int mxc_packed_sizes(const mxc_format *fmt, int64_t tokens, int64_t hidden,
                     size_t *code_bytes, size_t *scale_bytes);

/* Effective bits per element, b + s/block (Model Evaluation; Table 1; Table 3 caption).
 * Returns a negative value for an unsupported format. */
double mxc_effective_bits(const mxc_format *fmt);

/* Compress one partial (Method, "Communication Compression").
 *   x_bf16 : device, bf16 [tokens x hidden]
 *   codes  : device, out, packed codes (mxc_packed_sizes code_bytes)
 *   scales : device, out, scale bytes (scale_bytes) */
int mxc_quantize(const mxc_format *fmt, const void *x_bf16, int64_t tokens, int64_t hidden,
                 void *codes, void *scales, void *hip_stream);

/* The same for n (1..32) partials of identical shape in one launch.  x_bf16/codes/scales are
 * host arrays of n device pointers. */
int mxc_quantize_batched(const mxc_format *fmt, int n, const void *const *x_bf16,
                         int64_t tokens, int64_t hidden, void *const *codes,
                         void *const *scales, void *hip_stream);

/* Decompress the tp partials and add them (Profiling: decompress, then a plain sum).
 * out[t,h] = (((d_0 + d_1) + d_2) + ...) with binary32 adds in rank order, d_r the exactly
 * decoded value of rank r (a scale byte 255 decodes its block to NaN when s = 8).
 *   codes, scales : host arrays of tp device pointers
 *   out           : device, [tokens x hidden] of out_dtype (MXC_F32, or MXC_BF16 = that sum
 *                   rounded to nearest even; NaN becomes 0x7FC0)
 * Speed, not correctness: the kernel reads all tp code arrays at the same offset at the same
 * time, and arrays that lie a large power of two apart (eight 16 MiB arrays allocated back to
 * back) cost up to 7 % against the layout an all-gather leaves behind (rank r's codes followed
 * by its scales, the ranks back to back). */
int mxc_dequant_reduce(const mxc_format *fmt, int tp, const void *const *codes,
                       const void *const *scales, int64_t tokens, int64_t hidden, void *out,
                       int out_dtype, void *hip_stream);

/* The reduction as the paper's Profiling section words it: a worker decompresses the partials
 * of the N-1 other workers and adds its own partial uncompressed.  Like mxc_dequant_reduce, but
 * the term of rank own_rank (0..tp-1) is read from own_x_bf16 (device, bf16 [tokens x hidden],
 * exact in binary32) instead of being decoded; codes[own_rank] / scales[own_rank] are not read
 * and may be NULL.  The order of the adds is still rank order, so the result differs between
 * ranks only through which term is exact (and, with scales narrower than 8 bits, in blocks that
 * held an Inf or NaN: rule 5). */
int mxc_dequant_reduce_own(const mxc_format *fmt, int tp, int own_rank, const void *own_x_bf16,
                           const void *const *codes, const void *const *scales, int64_t tokens,
                           int64_t hidden, void *out, int out_dtype, void *hip_stream);

/* Quantize rows [chunk*tokens/tp, (chunk+1)*tokens/tp) of the reduced tensor (extension, see
 * top).  `reduced` is the whole [tokens x hidden] tensor of in_dtype (MXC_F32 or MXC_BF16);
 * codes_chunk / scales_chunk receive the packed arrays of a [tokens/tp x hidden] tensor. */
int mxc_requantize_chunk(const mxc_format *fmt, const void *reduced, int in_dtype,
                         int64_t tokens, int64_t hidden, int tp, int chunk, void *codes_chunk,
                         void *scales_chunk, void *hip_stream);

/* Fused form of the reduce-scatter leg (extension): exactly the result of
 *   mxc_dequant_reduce(fmt, tp, codes, scales, tokens, hidden, tmp, MXC_F32) followed by
 *   mxc_requantize_chunk(fmt, tmp, MXC_F32, tokens, hidden, 1, 0, codes_out, scales_out)
 * bit for bit, without the binary32 tensor ever reaching memory.  Here [tokens x hidden] is the
 * row chunk a rank owns and codes/scales are the tp compressed copies of that chunk it received
 * (host arrays of tp device pointers); codes_out/scales_out receive the packed arrays of the
 * re-quantized sum.  Requires tokens*hidden to be a multiple of 32 (always true for block 32),
 * MXC_ERR_SHAPE otherwise. */
int mxc_dequant_reduce_requantize(const mxc_format *fmt, int tp, const void *const *codes,
                                  const void *const *scales, int64_t tokens, int64_t hidden,
                                  void *codes_out, void *scales_out, void *hip_stream);

/* Measurement aid: copy `bytes` (a multiple of 16, both pointers 16-byte aligned) from src to
 * dst on the device with nontemporal 128-bit loads and stores, one per lane.  Its rate is the
 * practical ceiling the codec kernels are compared with. */
int mxc_copy_probe(void *dst, const void *src, size_t bytes, void *hip_stream);

/* Measurement aid: arm a pair of HIP events (hipEvent_t passed as void*, created by the caller with
 * timing enabled; either may be NULL) for the calling thread.  The next kernel this thread
 * launches through any entry point above stamps start_event when the kernel begins and
 * stop_event when it ends, from the dispatch's own timestamps, so hipEventElapsedTime between
 * them is the kernel's duration without the launch gap, and no extra packet enters the stream.
 * The pair is used once and then forgotten; a call that fails validation launches nothing and
 * leaves it armed; a valid call on an empty tensor launches nothing and disarms it; (NULL, NULL)
 * disarms.  Do not arm events for launches under stream capture.
 * Always returns MXC_OK. */
int mxc_time_next_launch(void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* MXC_H */
