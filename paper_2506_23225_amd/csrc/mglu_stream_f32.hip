// The streaming kernels for f32 elements (see mglu_stream_impl.hpp).
#include "mglu_stream_impl.hpp"

namespace mglu {

hipError_t launch_stream_f32(const StreamParams &p, int mode, hipStream_t stream)
{
    return launch_stream_t<F32Traits>(p, kElemF32, mode, stream);
}

}  // namespace mglu
