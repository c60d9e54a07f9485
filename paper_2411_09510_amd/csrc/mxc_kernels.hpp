// Device code of the mxc library for gfx950 (wave64): every kernel, through the headers below.
#pragma once

#include "mxc_common.hpp"
#include "mxc_quantize.hpp"
#include "mxc_reduce.hpp"

namespace mxc {

// ---------------------------------------------------------------------------------------------
// Plain 128-bit copy, the practical bandwidth ceiling the codec kernels are compared with.
template <int U, bool NT>
__global__ __launch_bounds__(kThreads) void copy_kernel(u32x4 *dst, const u32x4 *src, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * (size_t)(kThreads * U) + threadIdx.x;
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = base + (size_t)u * kThreads;
        if (i < n16) v[u] = ld<NT>(src + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const size_t i = base + (size_t)u * kThreads;
        if (i < n16) st<NT>(dst + i, v[u]);
    }
}

}  // namespace mxc
