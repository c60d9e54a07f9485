// Kernels behind mxc::host::quantize_bf16 (see mxc_dispatch.hpp).
#include "mxc_dispatch.hpp"

namespace mxc {
namespace host {

int quantize_bf16(const mxc_format *f, const QuantArgs &a, int n, hipStream_t st)
{
    return quantize_any<false>(f, a, n, st);
}

}  // namespace host
}  // namespace mxc
