// The MFMA-tiled kernel for bf16 elements (see mglu_prefill_impl.hpp).
#include "mglu_prefill_impl.hpp"

namespace mglu {

hipError_t launch_prefill_bf16(const PrefillParams &p, int mode, hipStream_t stream)
{
    return launch_prefill_t<Bf16Traits>(p, mode, stream);
}

}  // namespace mglu
