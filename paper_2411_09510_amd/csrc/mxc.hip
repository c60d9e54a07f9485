// Host side of the mxc C ABI: argument validation and kernel dispatch.  See include/mxc.h for
// the contract of every entry point.
#include "mxc_dispatch.hpp"

namespace mxc {
namespace host {

thread_local hipEvent_t t_start = nullptr, t_stop = nullptr;

}  // namespace host
}  // namespace mxc

namespace {

using namespace mxc;
using namespace mxc::host;

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

// A valid call on an empty tensor: nothing to launch, so events armed for "the next launch" would
// otherwise stamp some later, unrelated kernel.
int empty_ok()
{
    disarm();
    return MXC_OK;
}

bool aligned(const void *p, size_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

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
    if (a.units == 0) return empty_ok();
    for (int i = 0; i < 32; ++i) {
        const int k = i < n ? i : 0;
        a.x[i] = x[k];
        a.codes[i] = codes[k];
        a.scales[i] = scales[k];
    }
    a.sf = scale_fmt(fmt);
    hipStream_t st = (hipStream_t)hip_stream;
    return src32 ? quantize_f32(fmt, a, n, st) : quantize_bf16(fmt, a, n, st);
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

const char *mxc_version(void) { return "mxc 0.2 gfx950"; }

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
    if (a.units == 0) return empty_ok();
    a.out = out;
    return out_dtype == MXC_BF16 ? reduce_to_bf16(fmt, a, (hipStream_t)hip_stream)
                                 : reduce_to_f32(fmt, a, (hipStream_t)hip_stream);
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
    if (a.units == 0) return empty_ok();
    a.out = out;
    return out_dtype == MXC_BF16 ? reduce_own_to_bf16(fmt, a, (hipStream_t)hip_stream)
                                 : reduce_own_to_f32(fmt, a, (hipStream_t)hip_stream);
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
    if (a.units == 0) return empty_ok();
    a.codes_out = codes_out;
    a.scales_out = scales_out;
    return reduce_requantize(fmt, a, (hipStream_t)hip_stream);
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
    if (bytes == 0) return empty_ok();
    const size_t n16 = bytes / 16;
    return launch(copy_kernel<kCopyU, true>, dim3(grid_for(n16, kCopyU)), (hipStream_t)hip_stream,
                  (u32x4 *)dst, (const u32x4 *)src, n16);
}

int mxc_time_next_launch(void *start_event, void *stop_event)
{
    t_start = (hipEvent_t)start_event;
    t_stop = (hipEvent_t)stop_event;
    return MXC_OK;
}

}  // extern "C"
