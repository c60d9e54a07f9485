// Host-side plumbing shared by the library's translation units: launch shapes, the one function
// through which every kernel is enqueued, and the format dispatch.  The kernels of each family
// (quantize from bf16, quantize from binary32, the four reduce variants, the fused form) are
// instantiated in a translation unit of their own so that they compile side by side.
#pragma once

#include "mxc.h"

#include "mxc_kernels.hpp"

#include <hip/hip_ext.h>

#include <type_traits>

namespace mxc {
namespace host {

// Launch shapes, chosen by measurement on MI355X (HBM-bound kernels: more, smaller waves and
// nontemporal loads stream best).
constexpr int kQuantU = 2;          // units per lane, quantize from bf16
constexpr int kQuantU32 = 1;        // units per lane, quantize from binary32 (LDS-transposed loads)
constexpr bool kQuantNTL = true, kQuantNTS = true;
// nontemporal stores: measured 5 % faster than plain ones whenever the outputs of successive
// calls do not all fit the 256 MB last-level cache
constexpr bool kReduceNTL = true, kReduceNTS = true;
// Reduce kernel: ranks whose loads are issued together (rc) and whether the codes of a full tile
// are fetched through LDS (contiguous 128-bit loads that write LDS directly) or by each lane
// loading its own dwords, per code width and kernel form, each the fastest measured at the
// Llama-70B-shaped configuration (tp 8, 4096 x 8192).
struct TileShape {
    int rc;
    bool via_lds;
};
constexpr TileShape tile_shape(int code_bits, bool out_bf16, bool fused, bool own)
{
    if (code_bits == 4) return own ? TileShape{8, true} : TileShape{8, false};
    if (code_bits == 5) return own ? TileShape{8, false} : (out_bf16 || fused) ? TileShape{8, true} : TileShape{2, true};
    if (code_bits == 6) return (fused || own) ? TileShape{4, true} : TileShape{8, true};
    return {4, true};
}
// the copy probe: one 16-byte piece per lane, nontemporal (measured: 0.81 of peak against 0.77 with
// plain loads and stores, and against 0.67-0.77 for every form that moves more per wave)
constexpr int kCopyU = 1;
constexpr bool kHw = true;          // use the scaled-conversion instructions where exact

inline unsigned grid_for(size_t units, int per_lane)
{
    const size_t per_group = (size_t)kThreads * (size_t)per_lane;
    return (unsigned)((units + per_group - 1) / per_group);
}

// Events armed by mxc_time_next_launch for the calling thread; the next launch consumes them.
extern thread_local hipEvent_t t_start, t_stop;

// Drops the events armed by mxc_time_next_launch (used where a call ends without a launch).
inline void disarm()
{
    t_start = t_stop = nullptr;
}

// Every kernel of the library is enqueued here.  With armed events the launch goes through the
// extended launch call, which stamps them from the dispatch's own begin and end timestamps and
// adds no packet to the stream.  The status is the launch call's own return value: the thread's
// sticky error state, which other users of the runtime share, is neither read nor cleared.
template <class... Args>
int launch_wg(void (*kernel)(Args...), dim3 grid, dim3 block, hipStream_t st, Args... args)
{
    void *argv[] = {(void *)&args...};
    hipError_t err;
    if (t_start || t_stop) {
        err = hipExtLaunchKernel((const void *)kernel, grid, block, argv, 0, st, t_start, t_stop, 0);
        disarm();
    } else {
        err = hipLaunchKernel((const void *)kernel, grid, block, argv, 0, st);
    }
    return err == hipSuccess ? MXC_OK : MXC_ERR_HIP;
}

// Workgroups of kThreads threads.
template <class... Args>
int launch(void (*kernel)(Args...), dim3 grid, hipStream_t st, Args... args)
{
    return launch_wg(kernel, grid, dim3(kThreads), st, args...);
}

// Calls fn(Elem<x, y>{}, std::integral_constant<int, block>{}) for the format's element type and
// block size (both validated by the caller).
template <class Fn>
int for_block(int block, Fn fn)
{
    switch (block) {
    case 8: return fn(std::integral_constant<int, 8>{});
    case 16: return fn(std::integral_constant<int, 16>{});
    default: return fn(std::integral_constant<int, 32>{});
    }
}

template <class Fn>
int for_format(const mxc_format *f, Fn fn)
{
    auto with = [&](auto elem) { return for_block(f->block, [&](auto block) { return fn(elem, block); }); };
    switch (f->ebits * 10 + f->mbits) {
    case 11: return with(Elem<1, 1>{});
    case 12: return with(Elem<1, 2>{});
    case 13: return with(Elem<1, 3>{});
    case 14: return with(Elem<1, 4>{});
    case 21: return with(Elem<2, 1>{});
    case 22: return with(Elem<2, 2>{});
    case 23: return with(Elem<2, 3>{});
    case 31: return with(Elem<3, 1>{});
    case 32: return with(Elem<3, 2>{});
    default: return MXC_ERR_FORMAT;
    }
}

// One per translation unit of kernels.  All take validated arguments and enqueue one kernel.
int quantize_bf16(const mxc_format *f, const QuantArgs &a, int n, hipStream_t st);
int quantize_f32(const mxc_format *f, const QuantArgs &a, int n, hipStream_t st);
int reduce_to_f32(const mxc_format *f, const ReduceArgs &a, hipStream_t st);
int reduce_to_bf16(const mxc_format *f, const ReduceArgs &a, hipStream_t st);
int reduce_own_to_f32(const mxc_format *f, const ReduceArgs &a, hipStream_t st);
int reduce_own_to_bf16(const mxc_format *f, const ReduceArgs &a, hipStream_t st);
int reduce_requantize(const mxc_format *f, const ReduceArgs &a, hipStream_t st);

template <bool SRC32>
int quantize_any(const mxc_format *f, const QuantArgs &a, int n, hipStream_t st)
{
    return for_format(f, [&](auto elem, auto block) {
        using E = decltype(elem);
        constexpr int B = decltype(block)::value;
        constexpr int U = SRC32 ? kQuantU32 : kQuantU;
        return launch(quantize_kernel<E, B, SRC32, U, kQuantNTL, kQuantNTS, kHw, SRC32>,
                      dim3(grid_for(a.units, U), (unsigned)n), st, a);
    });
}

template <bool OUT_BF16, bool OWN>
int reduce_any(const mxc_format *f, const ReduceArgs &a, hipStream_t st)
{
    return for_format(f, [&](auto elem, auto block) {
        using E = decltype(elem);
        constexpr int B = decltype(block)::value;
        // half-chunk form: E2M1 codes, 6 to 8 ranks and a tensor of whole wave tiles (1024
        // elements = 128 units), up to the size where it stops paying
        if constexpr (kHalfFormOk<E>) {
            if (a.tp >= kHalfFormMinRanks && a.tp <= kFastRanks && a.units % 128 == 0 && a.units <= kHalfFormMaxUnits) {
                const size_t waves = a.units / 128;
                constexpr int per_wg = kHalfThreads / 64;
                return launch_wg(dequant_reduce_half_kernel<E, B, OUT_BF16, OWN, false, kReduceNTL, kReduceNTS>,
                                 dim3((unsigned)((waves + per_wg - 1) / per_wg)), dim3(kHalfThreads), st, a);
            }
        }
        // one lane per 32-element chunk (the last chunk may be shorter), output staged through LDS
        const size_t chunks = (a.units + 3) / 4;
        const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads));
        constexpr TileShape ts = tile_shape(E::bits, OUT_BF16, false, OWN);
        return launch(dequant_reduce_tile_kernel<E, B, OUT_BF16, ts.rc, kReduceNTL, kReduceNTS, kHw,
                                                 false, OWN, kThreads, ts.via_lds>,
                      grid, st, a);
    });
}

}  // namespace host
}  // namespace mxc
