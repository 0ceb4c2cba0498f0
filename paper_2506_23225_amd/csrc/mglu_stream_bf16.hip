// The streaming kernels for bf16 elements (see mglu_stream_impl.hpp).
#include "mglu_stream_impl.hpp"

namespace mglu {

hipError_t launch_stream_bf16(const StreamParams &p, int mode, hipStream_t stream)
{
    return launch_stream_t<Bf16Traits>(p, kElemBf16, mode, stream);
}

}  // namespace mglu
