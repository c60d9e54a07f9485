// Kernels behind mxc::host::reduce_to_f32 (see mxc_dispatch.hpp).
#include "mxc_dispatch.hpp"

namespace mxc {
namespace host {

int reduce_to_f32(const mxc_format *f, const ReduceArgs &a, hipStream_t st)
{
    return reduce_any<false, false>(f, a, st);
}

}  // namespace host
}  // namespace mxc
