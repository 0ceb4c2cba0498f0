// One-time set-up kernels: re-tile W and bit-pack the masks into the order the MGLU
// kernels stream them in (formats: see mglu_common.hpp).
//
// Paper: section "FlashMGLU", item "Packs mask bits" -- the n_m mask bits of a weight
// element are combined so that one load brings all mask information for a block of
// weights.  The paper spends one 8-bit integer per element whatever n_m is; here
// exactly n_m (rounded up to 1, 2, 4, 8) bits per element are stored, the figure its
// memory-load table counts, and their order is the register order of the consuming
// lane.  Masks and weights are fixed at inference, so none of this is on the
// per-token path.
#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

namespace mglu {

// One thread writes one 16-byte fragment (LANE_K consecutive k of one column).
template <typename Tr, typename elem_t>
__global__ __launch_bounds__(256) void pack_weights_kernel(PackParams p)
{
    const long total = (long)p.NB * p.NC * Tr::TILES * kWave;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int lane = (int)(gid % kWave);
    long rest = gid / kWave;
    const int t = (int)(rest % Tr::TILES);
    rest /= Tr::TILES;
    const int kc = (int)(rest % p.NC);
    const int jb = (int)(rest / p.NC);
    const int j = jb * kColBlock + (lane & 15);
    const int k0 = kc * kChunkK + t * Tr::TILE_K + (lane >> 4) * Tr::LANE_K;
    const elem_t *src = static_cast<const elem_t *>(p.src);
    elem_t v[Tr::LANE_K];
#pragma unroll
    for (int e = 0; e < Tr::LANE_K; ++e) {
        const int k = k0 + e;
        elem_t w = 0;
        if (j < p.d && k < p.h) w = p.nk ? src[(long)j * p.h + k] : src[(long)k * p.d + j];
        v[e] = w;
    }
    elem_t *dst = static_cast<elem_t *>(p.dst) + gid * Tr::LANE_K;
#pragma unroll
    for (int e = 0; e < Tr::LANE_K; ++e) dst[e] = v[e];
}

// One thread builds the NMP mask words of one lane of one chunk.
template <typename Tr, int NMP>
__global__ __launch_bounds__(256) void pack_masks_kernel(PackParams p)
{
    const long total = (long)p.NB * p.NC * kWave;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int lane = (int)(gid % kWave);
    const long rest = gid / kWave;
    const int kc = (int)(rest % p.NC);
    const int jb = (int)(rest / p.NC);
    const int j = jb * kColBlock + (lane & 15);
    const uint8_t *src = static_cast<const uint8_t *>(p.src);
    const long plane = (long)p.h * p.d;

    uint32_t words[NMP];
#pragma unroll
    for (int w = 0; w < NMP; ++w) words[w] = 0u;

#pragma unroll
    for (int t = 0; t < Tr::TILES; ++t) {
#pragma unroll
        for (int e = 0; e < Tr::LANE_K; ++e) {
            const int k = kc * kChunkK + t * Tr::TILE_K + (lane >> 4) * Tr::LANE_K + e;
            if (j >= p.d || k >= p.h) continue;
            const long off = p.nk ? (long)j * p.h + k : (long)k * p.d + j;
#pragma unroll
            for (int i = 0; i < NMP; ++i) {
                if (i >= p.n_masks) break;
                const uint32_t bit = src[i * plane + off] != 0 ? 1u : 0u;
                if constexpr (Tr::ELEM_BYTES == 2) {
                    words[Tr::template mask_word<NMP>(t, e >> 1, i)] |=
                        bit << (Tr::template mask_bit<NMP>(t, e >> 1, i) + 16 * (e & 1));
                } else {
                    const int lin = (4 * t + e) * NMP + i;         // element E = 4t + e
                    words[lin >> 5] |= bit << (lin & 31);
                }
            }
        }
    }
    // 16 bytes per lane per wavefront load: with 8 or 16 masks the lane's words go to NMP / 4 pieces
    // of 1 KiB of the chunk's mask block (words 0-3, then words 4-7, ...), so each load is one contiguous run
    if (NMP >= 8) {
        uint32_t *dst = static_cast<uint32_t *>(p.dst) + (gid / kWave) * (kWave * NMP) + lane * 4;
#pragma unroll
        for (int w = 0; w < NMP; ++w) dst[(w / 4) * (kWave * 4) + (w % 4)] = words[w];
    } else {
        uint32_t *dst = static_cast<uint32_t *>(p.dst) + gid * NMP;
#pragma unroll
        for (int w = 0; w < NMP; ++w) dst[w] = words[w];
    }
}

// Planar format: one thread builds, for one lane of one chunk, the word of every mask: bit
// Tr::planar_bit(t, e) of mask i's word = M_i at the lane's element (t, e).  The words of one mask of
// one column block are contiguous over the chunks: [jb][i][kc][lane].
template <typename Tr>
__global__ __launch_bounds__(256) void pack_masks_planar_kernel(PackParams p)
{
    const long total = (long)p.NB * p.NC * kWave;
    const long gid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= total) return;
    const int lane = (int)(gid % kWave);
    const long rest = gid / kWave;
    const int kc = (int)(rest % p.NC);
    const int jb = (int)(rest / p.NC);
    const int j = jb * kColBlock + (lane & 15);
    const uint8_t *src = static_cast<const uint8_t *>(p.src);
    const long plane = (long)p.h * p.d;
    uint32_t *dst = static_cast<uint32_t *>(p.dst);
    for (int i = 0; i < p.n_masks; ++i) {
        uint32_t word = 0u;
#pragma unroll
        for (int t = 0; t < Tr::TILES; ++t) {
#pragma unroll
            for (int e = 0; e < Tr::LANE_K; ++e) {
                const int k = kc * kChunkK + t * Tr::TILE_K + (lane >> 4) * Tr::LANE_K + e;
                if (j >= p.d || k >= p.h) continue;
                const long off = p.nk ? (long)j * p.h + k : (long)k * p.d + j;
                word |= (src[i * plane + off] != 0 ? 1u : 0u) << Tr::planar_bit(t, e);
            }
        }
        dst[(((long)jb * p.n_masks + i) * p.NC + kc) * kWave + lane] = word;
    }
}

hipError_t launch_pack_masks_planar(const PackParams &p, int elem, hipStream_t stream)
{
    const long total = (long)p.NB * p.NC * kWave;
    const dim3 grid((unsigned)ceil_div(total, 256)), block(256);
    if (elem == kElemF32) hipLaunchKernelGGL((pack_masks_planar_kernel<F32Traits>), grid, block, 0, stream, p);
    else hipLaunchKernelGGL((pack_masks_planar_kernel<Bf16Traits>), grid, block, 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_pack_weights(const PackParams &p, int elem, hipStream_t stream)
{
    const bool is_f32 = elem == kElemF32;   // bf16 and fp16 are both moved as 16-bit words
    const int tiles = is_f32 ? F32Traits::TILES : Bf16Traits::TILES;
    const long total = (long)p.NB * p.NC * tiles * kWave;
    const unsigned blocks = (unsigned)ceil_div(total, 256);
    if (is_f32)
        hipLaunchKernelGGL((pack_weights_kernel<F32Traits, float>), dim3(blocks), dim3(256), 0, stream, p);
    else
        hipLaunchKernelGGL((pack_weights_kernel<Bf16Traits, uint16_t>), dim3(blocks), dim3(256), 0, stream, p);
    return hipGetLastError();
}

template <typename Tr>
static hipError_t launch_pack_masks_t(const PackParams &p, hipStream_t stream)
{
    const long total = (long)p.NB * p.NC * kWave;
    const dim3 grid((unsigned)ceil_div(total, 256)), block(256);
    switch (round_up_masks(p.n_masks)) {
    case 1: hipLaunchKernelGGL((pack_masks_kernel<Tr, 1>), grid, block, 0, stream, p); break;
    case 2: hipLaunchKernelGGL((pack_masks_kernel<Tr, 2>), grid, block, 0, stream, p); break;
    case 4: hipLaunchKernelGGL((pack_masks_kernel<Tr, 4>), grid, block, 0, stream, p); break;
    case 8: hipLaunchKernelGGL((pack_masks_kernel<Tr, 8>), grid, block, 0, stream, p); break;
    default: hipLaunchKernelGGL((pack_masks_kernel<Tr, 16>), grid, block, 0, stream, p); break;
    }
    return hipGetLastError();
}

hipError_t launch_pack_masks(const PackParams &p, int elem, hipStream_t stream)
{
    const bool is_f32 = elem == kElemF32;   // the mask words of bf16 and fp16 are laid out alike
    return is_f32 ? launch_pack_masks_t<F32Traits>(p, stream) : launch_pack_masks_t<Bf16Traits>(p, stream);
}

}  // namespace mglu
