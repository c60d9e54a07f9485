// Host side of the mxc C ABI: argument validation and kernel dispatch.  See include/mxc.h for
// the contract of every entry point.
#include "mxc.h"

#include "mxc_kernels.hpp"

#include <hip/hip_ext.h>

namespace {

using namespace mxc;

bool format_ok(const mxc_format *f)
{
    if (!f) return false;
    if (f->ebits < 1 || f->ebits > 3 || f->mbits < 1 || f->mbits > 4) return false;
    const int b = 1 + f->ebits + f->mbits;
    if (b < 3 || b > 6) return false;
    if (f->block != 8 && f->block != 16 && f->block != 32) return false;
    if (f->scale_bits < 4 || f->scale_bits > 8) return false;
    return true;
}

ScaleFmt scale_fmt(const mxc_format *f)
{
    ScaleFmt s;
    s.sbits = f->scale_bits;
    s.sbias = (1 << (f->scale_bits - 1)) - 1;
    s.smax = f->scale_bits == 8 ? 254 : (1 << f->scale_bits) - 1;
    s.nonfinite = f->scale_bits == 8 ? 255 : s.smax;
    s.has_nan = f->scale_bits == 8 ? 1 : 0;
    return s;
}

// tokens*hidden as a number of 8-element units, or a negative status.
int shape_units(const mxc_format *f, int64_t tokens, int64_t hidden, size_t *units)
{
    if (tokens < 0 || hidden <= 0 || hidden % f->block) return MXC_ERR_SHAPE;
    // 2^40 elements at most: keeps every byte offset in 64 bits and every grid below 2^31 groups
    if (tokens > 0 && hidden > (int64_t)((1ull << 40) / (uint64_t)tokens)) return MXC_ERR_SHAPE;
    *units = (size_t)tokens * (size_t)hidden / 8;
    return MXC_OK;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

// Launch shapes, chosen by measurement on MI355X (HBM-bound kernels: more, smaller waves and
// nontemporal loads stream best).
constexpr int kQuantU = 2;          // units per lane, quantize from bf16
constexpr int kQuantU32 = 1;        // units per lane, quantize from binary32 (LDS-transposed loads)
constexpr bool kQuantNTL = true, kQuantNTS = true;
constexpr int kReduceU = 4;         // units per lane, dequant-reduce
constexpr int kReduceRC = 8;        // ranks loaded together, unit form
// nontemporal stores: measured 5 % faster than plain ones whenever the outputs of successive
// calls do not all fit the 256 MB last-level cache
constexpr bool kReduceNTL = true, kReduceNTS = true;
// ranks loaded together, tile form (measured: 4 is best or within noise of best for 4-, 5- and
// 6-bit codes)
template <class E> constexpr int tile_rc() { return 4; }
constexpr int kCopyU = 1;
constexpr bool kHw = true;          // use the scaled-conversion instructions where exact

unsigned grid_for(size_t units, int per_lane)
{
    const size_t per_group = (size_t)kThreads * (size_t)per_lane;
    return (unsigned)((units + per_group - 1) / per_group);
}

// Events armed by mxc_time_next_launch for the calling thread; the next launch consumes them.
thread_local hipEvent_t t_start = nullptr, t_stop = nullptr;

// Every kernel of the library is enqueued here.  With armed events the launch goes through the
// extended launch call, which stamps them from the dispatch's own begin and end timestamps and
// adds no packet to the stream.
template <class... Args>
int launch(void (*kernel)(Args...), dim3 grid, hipStream_t st, Args... args)
{
    if (t_start || t_stop) {
        hipExtLaunchKernelGGL(kernel, grid, dim3(kThreads), 0, st, t_start, t_stop, 0, args...);
        t_start = t_stop = nullptr;
    } else {
        hipLaunchKernelGGL(kernel, grid, dim3(kThreads), 0, st, args...);
    }
    return hipGetLastError() == hipSuccess ? MXC_OK : MXC_ERR_HIP;
}

template <class E, int B, bool SRC32>
int launch_quantize(const QuantArgs &a, int n, hipStream_t st)
{
    constexpr int U = SRC32 ? kQuantU32 : kQuantU;
    return launch(quantize_kernel<E, B, SRC32, U, kQuantNTL, kQuantNTS, kHw, SRC32>,
                  dim3(grid_for(a.units, U), (unsigned)n), st, a);
}

template <class E, bool SRC32>
int quantize_by_block(int block, const QuantArgs &a, int n, hipStream_t st)
{
    switch (block) {
    case 8: return launch_quantize<E, 8, SRC32>(a, n, st);
    case 16: return launch_quantize<E, 16, SRC32>(a, n, st);
    default: return launch_quantize<E, 32, SRC32>(a, n, st);
    }
}

template <bool SRC32>
int quantize_by_format(const mxc_format *f, const QuantArgs &a, int n, hipStream_t st)
{
    switch (f->ebits * 10 + f->mbits) {
    case 11: return quantize_by_block<Elem<1, 1>, SRC32>(f->block, a, n, st);
    case 12: return quantize_by_block<Elem<1, 2>, SRC32>(f->block, a, n, st);
    case 13: return quantize_by_block<Elem<1, 3>, SRC32>(f->block, a, n, st);
    case 14: return quantize_by_block<Elem<1, 4>, SRC32>(f->block, a, n, st);
    case 21: return quantize_by_block<Elem<2, 1>, SRC32>(f->block, a, n, st);
    case 22: return quantize_by_block<Elem<2, 2>, SRC32>(f->block, a, n, st);
    case 23: return quantize_by_block<Elem<2, 3>, SRC32>(f->block, a, n, st);
    case 31: return quantize_by_block<Elem<3, 1>, SRC32>(f->block, a, n, st);
    case 32: return quantize_by_block<Elem<3, 2>, SRC32>(f->block, a, n, st);
    default: return MXC_ERR_FORMAT;
    }
}

template <class E, int B, bool OUT_BF16, bool OWN>
int launch_reduce_as(const ReduceArgs &a, hipStream_t st)
{
    if (a.units % 4 == 0) {
        // whole 32-element chunks: one lane per chunk, output staged through LDS
        const size_t chunks = a.units / 4;
        const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads));
        return launch(dequant_reduce_tile_kernel<E, B, OUT_BF16, tile_rc<E>(), kReduceNTL,
                                                 kReduceNTS, kHw, false, OWN>,
                      grid, st, a);
    } else {
        // sizes that are not a multiple of 32 elements (only possible with blocks of 8 or 16)
        const dim3 grid(grid_for(a.units, kReduceU));
        return launch(dequant_reduce_kernel<E, B, OUT_BF16, kReduceU, kReduceRC, kReduceNTL,
                                            kReduceNTS, kHw, OWN>,
                      grid, st, a);
    }
}

template <class E, int B>
int launch_reduce(const ReduceArgs &a, bool out_bf16, hipStream_t st)
{
    const bool own = a.own_rank >= 0;
    if (out_bf16) return own ? launch_reduce_as<E, B, true, true>(a, st)
                             : launch_reduce_as<E, B, true, false>(a, st);
    return own ? launch_reduce_as<E, B, false, true>(a, st)
               : launch_reduce_as<E, B, false, false>(a, st);
}

template <class E, int B>
int launch_fused(const ReduceArgs &a, hipStream_t st)
{
    const size_t chunks = a.units / 4;
    const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads));
    // no LDS tile and a read-dominated stream: all eight ranks' loads in flight at once
    return launch(dequant_reduce_tile_kernel<E, B, false, 8, kReduceNTL, kQuantNTS, kHw, true>, grid,
                  st, a);
}

template <class E>
int fused_by_block(int block, const ReduceArgs &a, hipStream_t st)
{
    switch (block) {
    case 8: return launch_fused<E, 8>(a, st);
    case 16: return launch_fused<E, 16>(a, st);
    default: return launch_fused<E, 32>(a, st);
    }
}

int fused_by_format(const mxc_format *f, const ReduceArgs &a, hipStream_t st)
{
    switch (f->ebits * 10 + f->mbits) {
    case 11: return fused_by_block<Elem<1, 1>>(f->block, a, st);
    case 12: return fused_by_block<Elem<1, 2>>(f->block, a, st);
    case 13: return fused_by_block<Elem<1, 3>>(f->block, a, st);
    case 14: return fused_by_block<Elem<1, 4>>(f->block, a, st);
    case 21: return fused_by_block<Elem<2, 1>>(f->block, a, st);
    case 22: return fused_by_block<Elem<2, 2>>(f->block, a, st);
    case 23: return fused_by_block<Elem<2, 3>>(f->block, a, st);
    case 31: return fused_by_block<Elem<3, 1>>(f->block, a, st);
    case 32: return fused_by_block<Elem<3, 2>>(f->block, a, st);
    default: return MXC_ERR_FORMAT;
    }
}

template <class E>
int reduce_by_block(int block, const ReduceArgs &a, bool out_bf16, hipStream_t st)
{
    switch (block) {
    case 8: return launch_reduce<E, 8>(a, out_bf16, st);
    case 16: return launch_reduce<E, 16>(a, out_bf16, st);
    default: return launch_reduce<E, 32>(a, out_bf16, st);
    }
}

int reduce_by_format(const mxc_format *f, const ReduceArgs &a, bool out_bf16, hipStream_t st)
{
    switch (f->ebits * 10 + f->mbits) {
    case 11: return reduce_by_block<Elem<1, 1>>(f->block, a, out_bf16, st);
    case 12: return reduce_by_block<Elem<1, 2>>(f->block, a, out_bf16, st);
    case 13: return reduce_by_block<Elem<1, 3>>(f->block, a, out_bf16, st);
    case 14: return reduce_by_block<Elem<1, 4>>(f->block, a, out_bf16, st);
    case 21: return reduce_by_block<Elem<2, 1>>(f->block, a, out_bf16, st);
    case 22: return reduce_by_block<Elem<2, 2>>(f->block, a, out_bf16, st);
    case 23: return reduce_by_block<Elem<2, 3>>(f->block, a, out_bf16, st);
    case 31: return reduce_by_block<Elem<3, 1>>(f->block, a, out_bf16, st);
    case 32: return reduce_by_block<Elem<3, 2>>(f->block, a, out_bf16, st);
    default: return MXC_ERR_FORMAT;
    }
}

int quantize_common(const mxc_format *fmt, int n, const void *const *x, bool src32,
                    int64_t tokens, int64_t hidden, void *const *codes, void *const *scales,
                    void *hip_stream)
{
    if (!fmt || !x || !codes || !scales) return MXC_ERR_NULL;
    if (!format_ok(fmt)) return MXC_ERR_FORMAT;
    if (n < 1 || n > MXC_MAX_TP) return MXC_ERR_TP;
    QuantArgs a;
    int rc = shape_units(fmt, tokens, hidden, &a.units);
    if (rc != MXC_OK) return rc;
    for (int i = 0; i < n; ++i) {
        if (!x[i] || !codes[i] || !scales[i]) return MXC_ERR_NULL;
        if (!aligned(x[i], 16) || !aligned(codes[i], 16) || !aligned(scales[i], 4))
            return MXC_ERR_ALIGN;
    }
    if (a.units == 0) return MXC_OK;
    for (int i = 0; i < 32; ++i) {
        const int k = i < n ? i : 0;
        a.x[i] = x[k];
        a.codes[i] = codes[k];
        a.scales[i] = scales[k];
    }
    a.sf = scale_fmt(fmt);
    hipStream_t st = (hipStream_t)hip_stream;
    return src32 ? quantize_by_format<true>(fmt, a, n, st)
                 : quantize_by_format<false>(fmt, a, n, st);
}

// Validation shared by the reduce entry points; fills the pointer tables of `a`.
int reduce_args(const mxc_format *fmt, int tp, const void *const *codes, const void *const *scales,
                int64_t tokens, int64_t hidden, ReduceArgs *a, int own_rank = -1,
                const void *own_x = nullptr)
{
    if (!fmt || !codes || !scales) return MXC_ERR_NULL;
    if (!format_ok(fmt)) return MXC_ERR_FORMAT;
    if (tp < 1 || tp > MXC_MAX_TP) return MXC_ERR_TP;
    int rc = shape_units(fmt, tokens, hidden, &a->units);
    if (rc != MXC_OK) return rc;
    for (int r = 0; r < tp; ++r) {
        if (r == own_rank) continue;              // that rank's compressed arrays are not read
        if (!codes[r] || !scales[r]) return MXC_ERR_NULL;
        if (!aligned(codes[r], 16) || !aligned(scales[r], 4)) return MXC_ERR_ALIGN;
    }
    for (int r = 0; r < 32; ++r) {
        a->codes[r] = codes[r < tp ? r : 0];
        a->scales[r] = scales[r < tp ? r : 0];
    }
    a->own_rank = own_rank;
    a->own_x = own_x;
    a->out = nullptr;
    a->codes_out = nullptr;
    a->scales_out = nullptr;
    a->tp = tp;
    a->sf = scale_fmt(fmt);
    return MXC_OK;
}

}  // namespace

extern "C" {

const char *mxc_strerror(int status)
{
    switch (status) {
    case MXC_OK: return "ok";
    case MXC_ERR_NULL: return "a required pointer is NULL";
    case MXC_ERR_FORMAT: return "unsupported element, block or scale format";
    case MXC_ERR_SHAPE: return "bad shape (non-positive, hidden % block != 0, tokens % tp != 0 or too large)";
    case MXC_ERR_ALIGN: return "device pointer not aligned (16 bytes for tensors and codes, 4 for scales)";
    case MXC_ERR_TP: return "tp, chunk or batch count out of range";
    case MXC_ERR_HIP: return "HIP runtime refused the kernel launch";
    case MXC_ERR_DTYPE: return "unknown dtype";
    default: return "unknown mxc status";
    }
}

const char *mxc_version(void) { return "mxc 0.1 gfx950"; }

int mxc_packed_sizes(const mxc_format *fmt, int64_t tokens, int64_t hidden, size_t *code_bytes,
                     size_t *scale_bytes)
{
    if (!fmt) return MXC_ERR_NULL;
    if (!format_ok(fmt)) return MXC_ERR_FORMAT;
    size_t units;
    int rc = shape_units(fmt, tokens, hidden, &units);
    if (rc != MXC_OK) return rc;
    const size_t b = (size_t)(1 + fmt->ebits + fmt->mbits);
    if (code_bytes) *code_bytes = units * b;
    const size_t blocks = units * 8 / (size_t)fmt->block;
    if (scale_bytes)
        *scale_bytes = fmt->scale_bits == 8 ? blocks : (blocks * (size_t)fmt->scale_bits + 7) / 8;
    return MXC_OK;
}

double mxc_effective_bits(const mxc_format *fmt)
{
    if (!format_ok(fmt)) return -1.0;
    return (double)(1 + fmt->ebits + fmt->mbits) + (double)fmt->scale_bits / (double)fmt->block;
}

int mxc_quantize(const mxc_format *fmt, const void *x_bf16, int64_t tokens, int64_t hidden,
                 void *codes, void *scales, void *hip_stream)
{
    const void *xs[1] = {x_bf16};
    void *cs[1] = {codes};
    void *ss[1] = {scales};
    return quantize_common(fmt, 1, xs, false, tokens, hidden, cs, ss, hip_stream);
}

int mxc_quantize_batched(const mxc_format *fmt, int n, const void *const *x_bf16, int64_t tokens,
                         int64_t hidden, void *const *codes, void *const *scales,
                         void *hip_stream)
{
    return quantize_common(fmt, n, x_bf16, false, tokens, hidden, codes, scales, hip_stream);
}

int mxc_dequant_reduce(const mxc_format *fmt, int tp, const void *const *codes,
                       const void *const *scales, int64_t tokens, int64_t hidden, void *out,
                       int out_dtype, void *hip_stream)
{
    if (!out) return MXC_ERR_NULL;
    if (out_dtype != MXC_F32 && out_dtype != MXC_BF16)
        return (!fmt || !codes || !scales) ? MXC_ERR_NULL : MXC_ERR_DTYPE;
    ReduceArgs a;
    int rc = reduce_args(fmt, tp, codes, scales, tokens, hidden, &a);
    if (rc != MXC_OK) return rc;
    if (!aligned(out, 16)) return MXC_ERR_ALIGN;
    if (a.units == 0) return MXC_OK;
    a.out = out;
    return reduce_by_format(fmt, a, out_dtype == MXC_BF16, (hipStream_t)hip_stream);
}

int mxc_dequant_reduce_own(const mxc_format *fmt, int tp, int own_rank, const void *own_x_bf16,
                           const void *const *codes, const void *const *scales, int64_t tokens,
                           int64_t hidden, void *out, int out_dtype, void *hip_stream)
{
    if (!out || !own_x_bf16) return MXC_ERR_NULL;
    if (out_dtype != MXC_F32 && out_dtype != MXC_BF16)
        return (!fmt || !codes || !scales) ? MXC_ERR_NULL : MXC_ERR_DTYPE;
    if (tp >= 1 && tp <= MXC_MAX_TP && (own_rank < 0 || own_rank >= tp)) return MXC_ERR_TP;
    ReduceArgs a;
    int rc = reduce_args(fmt, tp, codes, scales, tokens, hidden, &a, own_rank, own_x_bf16);
    if (rc != MXC_OK) return rc;
    if (!aligned(out, 16) || !aligned(own_x_bf16, 16)) return MXC_ERR_ALIGN;
    if (a.units == 0) return MXC_OK;
    a.out = out;
    return reduce_by_format(fmt, a, out_dtype == MXC_BF16, (hipStream_t)hip_stream);
}

int mxc_dequant_reduce_requantize(const mxc_format *fmt, int tp, const void *const *codes,
                                  const void *const *scales, int64_t tokens, int64_t hidden,
                                  void *codes_out, void *scales_out, void *hip_stream)
{
    if (!codes_out || !scales_out) return MXC_ERR_NULL;
    ReduceArgs a;
    int rc = reduce_args(fmt, tp, codes, scales, tokens, hidden, &a);
    if (rc != MXC_OK) return rc;
    if (a.units % 4) return MXC_ERR_SHAPE;
    if (!aligned(codes_out, 16) || !aligned(scales_out, 4)) return MXC_ERR_ALIGN;
    if (a.units == 0) return MXC_OK;
    a.codes_out = codes_out;
    a.scales_out = scales_out;
    return fused_by_format(fmt, a, (hipStream_t)hip_stream);
}

int mxc_requantize_chunk(const mxc_format *fmt, const void *reduced, int in_dtype, int64_t tokens,
                         int64_t hidden, int tp, int chunk, void *codes_chunk, void *scales_chunk,
                         void *hip_stream)
{
    if (!fmt || !reduced || !codes_chunk || !scales_chunk) return MXC_ERR_NULL;
    if (!format_ok(fmt)) return MXC_ERR_FORMAT;
    if (in_dtype != MXC_F32 && in_dtype != MXC_BF16) return MXC_ERR_DTYPE;
    if (tp < 1 || tp > MXC_MAX_TP || chunk < 0 || chunk >= tp) return MXC_ERR_TP;
    if (tokens < 0 || tokens % tp) return MXC_ERR_SHAPE;
    size_t units;
    int rc = shape_units(fmt, tokens, hidden, &units);
    if (rc != MXC_OK) return rc;
    const int64_t rows = tokens / tp;
    const size_t elem = in_dtype == MXC_F32 ? 4 : 2;
    const char *src = (const char *)reduced + (size_t)chunk * (size_t)rows * (size_t)hidden * elem;
    const void *xs[1] = {src};
    void *cs[1] = {codes_chunk};
    void *ss[1] = {scales_chunk};
    if (!aligned(reduced, 16)) return MXC_ERR_ALIGN;
    return quantize_common(fmt, 1, xs, in_dtype == MXC_F32, rows, hidden, cs, ss, hip_stream);
}

int mxc_copy_probe(void *dst, const void *src, size_t bytes, void *hip_stream)
{
    if (!dst || !src) return MXC_ERR_NULL;
    if (bytes % 16) return MXC_ERR_SHAPE;
    if (!aligned(dst, 16) || !aligned(src, 16)) return MXC_ERR_ALIGN;
    if (bytes == 0) return MXC_OK;
    const size_t n16 = bytes / 16;
    return launch(copy_kernel<kCopyU, false>, dim3(grid_for(n16, kCopyU)), (hipStream_t)hip_stream,
                  (u32x4 *)dst, (const u32x4 *)src, n16);
}

int mxc_time_next_launch(void *start_event, void *stop_event)
{
    t_start = (hipEvent_t)start_event;
    t_stop = (hipEvent_t)stop_event;
    return MXC_OK;
}

}  // extern "C"
