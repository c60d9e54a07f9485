// Kernels behind mxc::host::reduce_to_bf16 (see mxc_dispatch.hpp).
#include "mxc_dispatch.hpp"

namespace mxc {
namespace host {

int reduce_to_bf16(const mxc_format *f, const ReduceArgs &a, hipStream_t st)
{
    return reduce_any<true, false>(f, a, st);
}

}  // namespace host
}  // namespace mxc
