// Kernels behind mxc::host::reduce_requantize: the fused dequant-reduce + requantize form.
#include "mxc_dispatch.hpp"

namespace mxc {
namespace host {

int reduce_requantize(const mxc_format *f, const ReduceArgs &a, hipStream_t st)
{
    return for_format(f, [&](auto elem, auto block) {
        using E = decltype(elem);
        constexpr int B = decltype(block)::value;
        // half-chunk form, as for the plain reduction
        if constexpr (kHalfFormOk<E>) {
            if (a.tp >= kHalfFormMinRanks && a.tp <= kFastRanks && a.units % 128 == 0 && a.units <= kHalfFormMaxUnits) {
                const size_t waves = a.units / 128;
                constexpr int per_wg = kHalfThreads / 64;
                return launch_wg(dequant_reduce_half_kernel<E, B, false, false, true, kReduceNTL, kQuantNTS>,
                                 dim3((unsigned)((waves + per_wg - 1) / per_wg)), dim3(kHalfThreads), st, a);
            }
        }
        const size_t chunks = a.units / 4;
        const dim3 grid((unsigned)((chunks + kThreads - 1) / kThreads));
        constexpr TileShape ts = tile_shape(E::bits, false, true, false);
        return launch(dequant_reduce_tile_kernel<E, B, false, ts.rc, kReduceNTL, kQuantNTS, kHw, true, false,
                                                 kThreads, ts.via_lds>,
                      grid, st, a);
    });
}

}  // namespace host
}  // namespace mxc
