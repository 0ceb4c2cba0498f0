// The MFMA-tiled kernel for f16 elements (see mglu_prefill_impl.hpp).
#include "mglu_prefill_impl.hpp"

namespace mglu {

hipError_t launch_prefill_f16(const PrefillParams &p, int mode, hipStream_t stream)
{
    return launch_prefill_t<F16Traits>(p, mode, stream);
}

}  // namespace mglu
