// Kernels behind mxc::host::quantize_f32 (see mxc_dispatch.hpp).
#include "mxc_dispatch.hpp"

namespace mxc {
namespace host {

int quantize_f32(const mxc_format *f, const QuantArgs &a, int n, hipStream_t st)
{
    return quantize_any<true>(f, a, n, st);
}

}  // namespace host
}  // namespace mxc
