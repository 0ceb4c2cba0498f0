// Router of the Top-K routed MGLU (appendix "Top-K Routing"): logits l = x W_r, keep the K largest
// per token, softmax over the kept ones, 0 elsewhere.  One wavefront per token; W_r is h x n_masks
// and tiny, so this is a few dot products, a butterfly reduction and a scalar tail.
#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

namespace mglu {

template <typename elem_t>
__device__ __forceinline__ float route_elem(const void *p, long i);
template <>
__device__ __forceinline__ float route_elem<float>(const void *p, long i) { return static_cast<const float *>(p)[i]; }
template <>
__device__ __forceinline__ float route_elem<uint16_t>(const void *p, long i)
{
    return bf16_bits_to_f32(static_cast<const uint16_t *>(p)[i]);
}
template <>
__device__ __forceinline__ float route_elem<_Float16>(const void *p, long i)
{
    return (float)static_cast<const _Float16 *>(p)[i];
}

template <typename elem_t>
__global__ __launch_bounds__(256) void route_topk_kernel(RouteParams p)
{
    const int lane = threadIdx.x & 63;
    const int tok = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (tok >= p.T) return;
    float logit[kMaxMasks];
#pragma unroll
    for (int i = 0; i < kMaxMasks; ++i) logit[i] = 0.f;
    for (int k = lane; k < p.h; k += kWave) {
        const float xv = route_elem<elem_t>(p.x, (long)tok * p.h + k);
#pragma unroll
        for (int i = 0; i < kMaxMasks; ++i)
            if (i < p.n_masks) logit[i] += xv * route_elem<elem_t>(p.wr, (long)k * p.n_masks + i);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1)
#pragma unroll
        for (int i = 0; i < kMaxMasks; ++i) logit[i] += __shfl_xor(logit[i], off, kWave);
    if (lane != 0) return;

    // K largest (on equal logits the lower index wins), then a softmax over them
    bool kept[kMaxMasks];
#pragma unroll
    for (int i = 0; i < kMaxMasks; ++i) kept[i] = false;
    float top = -INFINITY;
    for (int c = 0; c < p.k; ++c) {
        int best = -1;
        float best_v = -INFINITY;
#pragma unroll
        for (int i = 0; i < kMaxMasks; ++i)
            if (i < p.n_masks && !kept[i] && (best < 0 || logit[i] > best_v)) { best = i; best_v = logit[i]; }
#pragma unroll
        for (int i = 0; i < kMaxMasks; ++i)
            if (i == best) kept[i] = true;
        if (c == 0) top = best_v;
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxMasks; ++i)
        if (i < p.n_masks && kept[i]) sum += __expf(logit[i] - top);
#pragma unroll
    for (int i = 0; i < kMaxMasks; ++i)
        if (i < p.n_masks) p.weights[(long)tok * p.n_masks + i] = kept[i] ? __expf(logit[i] - top) / sum : 0.f;
}

hipError_t launch_route_topk(const RouteParams &p, int elem, hipStream_t stream)
{
    const dim3 grid((unsigned)ceil_div(p.T, 4)), block(256);
    if (elem == kElemF32) hipLaunchKernelGGL(route_topk_kernel<float>, grid, block, 0, stream, p);
    else if (elem == kElemF16) hipLaunchKernelGGL(route_topk_kernel<_Float16>, grid, block, 0, stream, p);
    else hipLaunchKernelGGL(route_topk_kernel<uint16_t>, grid, block, 0, stream, p);
    return hipGetLastError();
}

}  // namespace mglu
