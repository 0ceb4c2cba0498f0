// Entry point of the MFMA-tiled kernel: dispatch on the element type (the kernel is in
// mglu_prefill_impl.hpp, instantiated per element type in mglu_prefill_bf16.hip and _f16.hip).
#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

namespace mglu {

hipError_t launch_prefill_bf16(const PrefillParams &p, int mode, hipStream_t stream);
hipError_t launch_prefill_f16(const PrefillParams &p, int mode, hipStream_t stream);

hipError_t launch_prefill(const PrefillParams &p, int elem, int mode, hipStream_t stream)
{
    return elem == kElemF16 ? launch_prefill_f16(p, mode, stream) : launch_prefill_bf16(p, mode, stream);
}

}  // namespace mglu
