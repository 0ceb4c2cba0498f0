// The streaming kernels for f16 elements (see mglu_stream_impl.hpp).
#include "mglu_stream_impl.hpp"

namespace mglu {

hipError_t launch_stream_f16(const StreamParams &p, int mode, hipStream_t stream)
{
    return launch_stream_t<F16Traits>(p, kElemF16, mode, stream);
}

}  // namespace mglu
