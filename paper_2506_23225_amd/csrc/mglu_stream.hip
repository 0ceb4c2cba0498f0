// Entry points of the streaming kernels: dispatch on the element type (the kernels themselves are in
// mglu_stream_impl.hpp, instantiated per element type in mglu_stream_bf16.hip, _f16.hip, _f32.hip)
// and the read-bandwidth calibrator.
#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

namespace mglu {

hipError_t launch_stream_bf16(const StreamParams &p, int mode, hipStream_t stream);
hipError_t launch_stream_f16(const StreamParams &p, int mode, hipStream_t stream);
hipError_t launch_stream_f32(const StreamParams &p, int mode, hipStream_t stream);

hipError_t launch_stream(const StreamParams &p, int elem, int mode, hipStream_t stream)
{
    if (elem == kElemF32) return launch_stream_f32(p, mode, stream);
    if (elem == kElemF16) return launch_stream_f16(p, mode, stream);
    return launch_stream_bf16(p, mode, stream);
}

// ---- read-bandwidth calibrator: the same 16-byte-per-lane, 1 KiB-per-wavefront loads, nothing else ----
__global__ __launch_bounds__(512) void stream_read_kernel(const u32x4 *__restrict__ buf, long n16, uint32_t *sink)
{
    const long stride = (long)gridDim.x * blockDim.x;
    u32x4 a = {0, 0, 0, 0};
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        u32x4 v0 = __builtin_nontemporal_load(buf + i);
        u32x4 v1 = __builtin_nontemporal_load(buf + i + stride);
        u32x4 v2 = __builtin_nontemporal_load(buf + i + 2 * stride);
        u32x4 v3 = __builtin_nontemporal_load(buf + i + 3 * stride);
        a ^= v0 ^ v1 ^ v2 ^ v3;
    }
    for (; i < n16; i += stride) a ^= __builtin_nontemporal_load(buf + i);
    const uint32_t f = a.x ^ a.y ^ a.z ^ a.w;
    if (f == 0x9e3779b9u) atomicXor(sink + (threadIdx.x & 255), f);  // practically never: keeps the loads alive
}

hipError_t launch_stream_read(const void *buf, size_t bytes, uint32_t *sink, hipStream_t stream)
{
    const long n16 = (long)(bytes / 16);
    long blocks = ceil_div(n16, 512 * 4);
    if (blocks > 256 * 8) blocks = 256 * 8;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)blocks), dim3(512), 0, stream,
                       static_cast<const u32x4 *>(buf), n16, sink);
    return hipGetLastError();
}

}  // namespace mglu
