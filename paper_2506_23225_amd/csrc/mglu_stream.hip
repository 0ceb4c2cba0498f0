// Streaming MGLU kernel for decode and small batches (tokens <= 64): HBM-bound.
//
// Paper: section "FlashMGLU", Alg. 1 (split-K matrix-vector product with packed
// masks).  Kept from it: W and the packed mask words are read once, the unmasked
// sum and one sum per mask are accumulated together in registers, the value
// branch comes from the complement, partial sums of a K split are combined on
// chip.  Different from it, for gfx950:
//   - the multiply-accumulates run on the matrix cores (v_mfma_f32_16x16x32_bf16,
//     tokens padded to 16 per tile), so the vector ALUs only prepare operands;
//   - a mask bit flips the sign of its weight element (one shift + one 3-input
//     bit-op per register pair and mask) instead of predicating an add; the gate
//     and value sums are recovered as (t -/+ dsum)/2;
//   - the K split is across the wavefronts of one workgroup and is combined in a
//     fixed order through LDS -- no float atomics, bit-reproducible results;
//   - Swish, the gate*value products and the sum over masks are applied to the
//     reduced sums in registers and only `out` is written (Eq. 3).
//
// Work split: workgroup (jb, tg) owns output columns [16 jb, 16 jb + 16) for the
// token group tg of 16*TB tokens; its wavefronts take the chunks kc = wave, wave +
// nw, ... of that column block, so at any moment the workgroup reads one contiguous
// run of the packed weight stream.
#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

namespace mglu {

template <typename Tr, int NMP, int TB, int MODE>
struct Chunk {
    typename Tr::frag w[Tr::TILES];
    typename Tr::frag w2[MODE == kModeSwiglu ? Tr::TILES : 1];
    uint32_t m[NMP];
    typename Tr::frag x[TB][Tr::TILES];
};

template <typename Tr, int NMP, int TB, int MODE>
__global__ __launch_bounds__(512) void stream_kernel(StreamParams p)
{
    constexpr int SETS = (MODE == kModeSwiglu) ? 2 : 1 + NMP;
    constexpr long CHUNK_BYTES = (long)kColBlock * kChunkK * Tr::ELEM_BYTES;
    typedef typename Tr::frag frag;
    extern __shared__ f32x4 lds[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = blockDim.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int jb = blockIdx.x;
    const int tok0 = blockIdx.y * (16 * TB);

    const char *wbase = static_cast<const char *>(p.w) + (long)jb * p.NC * CHUNK_BYTES + lane * 16;
    const char *w2base = static_cast<const char *>(p.w2) + (long)jb * p.NC * CHUNK_BYTES + lane * 16;
    const uint32_t *mbase = p.m + ((long)jb * p.NC * kWave + lane) * NMP;

    bool tok_ok[TB];
    const char *xrow[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const int tok = tok0 + 16 * tb + r;
        tok_ok[tb] = tok < p.T;
        xrow[tb] = static_cast<const char *>(p.x) + (long)(tok_ok[tb] ? tok : 0) * p.h * Tr::ELEM_BYTES;
    }

    f32x4 acc[SETS][TB];
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[s][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    typedef Chunk<Tr, NMP, TB, MODE> chunk_t;

    auto load_chunk = [&](chunk_t &c, int kc) {
        const char *wp = wbase + (long)kc * CHUNK_BYTES;
#pragma unroll
        for (int t = 0; t < Tr::TILES; ++t)
            c.w[t] = __builtin_nontemporal_load(reinterpret_cast<const frag *>(wp + t * 1024));
        if constexpr (MODE == kModeSwiglu) {
            const char *wp2 = w2base + (long)kc * CHUNK_BYTES;
#pragma unroll
            for (int t = 0; t < Tr::TILES; ++t)
                c.w2[t] = __builtin_nontemporal_load(reinterpret_cast<const frag *>(wp2 + t * 1024));
        } else {
            const uint32_t *mp = mbase + (long)kc * kWave * NMP;
            if constexpr (NMP == 8) {
                u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(mp));
                u32x4 b = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(mp) + 1);
#pragma unroll
                for (int i = 0; i < 4; ++i) { c.m[i] = a[i]; c.m[4 + i] = b[i]; }
            } else if constexpr (NMP == 4) {
                u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(mp));
#pragma unroll
                for (int i = 0; i < 4; ++i) c.m[i] = a[i];
            } else if constexpr (NMP == 2) {
                u32x2 a = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(mp));
                c.m[0] = a.x; c.m[1] = a.y;
            } else {
                c.m[0] = __builtin_nontemporal_load(mp);
            }
        }
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
#pragma unroll
            for (int t = 0; t < Tr::TILES; ++t) {
                const int k0 = kc * kChunkK + t * Tr::TILE_K + q * Tr::LANE_K;
                frag v = frag{0, 0, 0, 0};
                if (tok_ok[tb] && k0 < p.h)
                    v = *reinterpret_cast<const frag *>(xrow[tb] + (long)k0 * Tr::ELEM_BYTES);
                c.x[tb][t] = v;
            }
    };

    auto compute = [&](const chunk_t &c) {
#pragma unroll
        for (int t = 0; t < Tr::TILES; ++t) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) acc[0][tb] = Tr::mma(c.w[t], c.x[tb][t], acc[0][tb]);
            if constexpr (MODE == kModeSwiglu) {
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) acc[1][tb] = Tr::mma(c.w2[t], c.x[tb][t], acc[1][tb]);
            } else {
#pragma unroll
                for (int i = 0; i < NMP; ++i) {
                    const frag wf = Tr::template flip<NMP>(c.w[t], c.m, t, i);
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) acc[1 + i][tb] = Tr::mma(wf, c.x[tb][t], acc[1 + i][tb]);
                }
            }
        }
    };

    // ---- stream this wavefront's chunks, one chunk of loads in flight ahead of the math ----
    {
        int kc = wave;
        if (kc < p.NC) {
            chunk_t cur, nxt;
            load_chunk(cur, kc);
            for (;;) {
                const int kn = kc + nw;
                const bool more = kn < p.NC;  // uniform over the wavefront
                if (more) load_chunk(nxt, kn);
                compute(cur);
                if (!more) break;
                cur = nxt;
                kc = kn;
            }
        }
    }

    // ---- combine the K split: wavefronts 1..nw-1 hand their sums to wavefront 0 through LDS,
    //      which adds them in wavefront order (fixed order => reproducible bits) -------------
    const int tc = (TB == 1) ? min(p.T - tok0, 16) : 16;  // token lanes that carry data
    if (nw > 1) {
        if (wave > 0 && r < tc) {
#pragma unroll
            for (int s = 0; s < SETS; ++s)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
                    lds[(((wave - 1) * SETS + s) * TB + tb) * (4 * tc) + q * tc + r] = acc[s][tb];
        }
        __syncthreads();
        if (wave == 0 && r < tc) {
            for (int w = 1; w < nw; ++w)
#pragma unroll
                for (int s = 0; s < SETS; ++s)
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
                        acc[s][tb] += lds[(((w - 1) * SETS + s) * TB + tb) * (4 * tc) + q * tc + r];
        }
    }
    if (wave != 0) return;

    // ---- epilogue on the reduced sums (Eq. 3): lane (r, q) holds token r, columns 4q..4q+3 ----
    const int j0 = jb * kColBlock + 4 * q;
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        if (!tok_ok[tb] || j0 >= p.d) continue;
        const long tok = tok0 + 16 * tb + r;
        const long o = tok * p.d + j0;
        const bool full = (j0 + 3 < p.d) && ((p.d & 3) == 0);
        if constexpr (MODE == kModeProjections) {
            const long plane = (long)p.T * p.d;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (j0 + c >= p.d) break;
                const float t = acc[0][tb][c];
                if (p.proj_t) p.proj_t[o + c] = t;
#pragma unroll
                for (int i = 0; i < NMP; ++i) {
                    if (i >= p.n_masks) break;
                    const float ds = acc[1 + i][tb][c];
                    if (p.proj_gate) p.proj_gate[i * plane + o + c] = gate_of(t, ds);
                    if (p.proj_value) p.proj_value[i * plane + o + c] = value_of(t, ds);
                }
            }
        } else {
            f32x4 y;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if constexpr (MODE == kModeSwiglu) {
                    y[c] = swish(acc[0][tb][c]) * acc[1][tb][c];
                } else {
                    const float t = acc[0][tb][c];
                    float sum = 0.f;
#pragma unroll
                    for (int i = 0; i < NMP; ++i) {
                        if (i >= p.n_masks) break;
                        const float ds = acc[1 + i][tb][c];
                        sum += swish(gate_of(t, ds)) * value_of(t, ds);
                    }
                    y[c] = sum;
                }
            }
            if (full) {
                Tr::store4(p.out, o, y);
            } else {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (j0 + c < p.d) Tr::store1(p.out, o + c, y[c]);
            }
        }
    }
}

// ---- host side --------------------------------------------------------------------------------

template <typename Tr, int NMP, int TB, int MODE>
static hipError_t launch_one(const StreamParams &p, int nw, size_t lds_bytes, dim3 grid, hipStream_t stream)
{
    auto kern = stream_kernel<Tr, NMP, TB, MODE>;
    if (lds_bytes > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, grid, dim3(nw * kWave), lds_bytes, stream, p);
    return hipGetLastError();
}

template <typename Tr, int NMP, int MODE>
static hipError_t launch_tb(const StreamParams &p, int tb, int nw, size_t lds, dim3 grid, hipStream_t s)
{
    // token blocks per workgroup are bounded by the 256-register budget: see stream_max_token_blocks
    constexpr bool kIsBf16 = Tr::ELEM_BYTES == 2;
    if (tb == 1) return launch_one<Tr, NMP, 1, MODE>(p, nw, lds, grid, s);
    if constexpr (kIsBf16) {
        if (tb == 2) return launch_one<Tr, NMP, 2, MODE>(p, nw, lds, grid, s);
        if constexpr (NMP <= 2) {
            if (tb == 4) return launch_one<Tr, NMP, 4, MODE>(p, nw, lds, grid, s);
        }
    }
    return hipErrorInvalidValue;
}

template <typename Tr, int MODE>
static hipError_t launch_nmp(const StreamParams &p, int nmp, int tb, int nw, size_t lds, dim3 grid, hipStream_t s)
{
    switch (nmp) {
    case 1: return launch_tb<Tr, 1, MODE>(p, tb, nw, lds, grid, s);
    case 2: return launch_tb<Tr, 2, MODE>(p, tb, nw, lds, grid, s);
    case 4: return launch_tb<Tr, 4, MODE>(p, tb, nw, lds, grid, s);
    default: return launch_tb<Tr, 8, MODE>(p, tb, nw, lds, grid, s);
    }
}

// Largest token block count per workgroup the register budget allows for this mask count.
int stream_max_token_blocks(int nmp, bool is_f32) { return is_f32 ? 1 : nmp <= 2 ? 4 : 2; }

hipError_t launch_stream(const StreamParams &p, bool is_f32, int mode, hipStream_t stream)
{
    const int nmp = (mode == kModeSwiglu) ? 1 : round_up_masks(p.n_masks);
    const int sets = (mode == kModeSwiglu) ? 2 : 1 + nmp;
    const int max_tb = stream_max_token_blocks(nmp, is_f32);
    const int blocks = (int)ceil_div(p.T, 16);
    const int tb = (blocks >= 4 && max_tb >= 4) ? 4 : (blocks >= 2 && max_tb >= 2) ? 2 : 1;
    const int tc = (tb == 1) ? (p.T < 16 ? p.T : 16) : 16;

    // wavefronts per workgroup: as many as there are chunks, at most 8, and the LDS hand-over must fit
    int nw = p.NC < 8 ? p.NC : 8;
    auto lds_bytes = [&](int n) { return (size_t)(n - 1) * sets * tb * 4 * tc * sizeof(f32x4); };
    while (nw > 1 && lds_bytes(nw) > 64 * 1024) nw >>= 1;
    const size_t lds = nw > 1 ? lds_bytes(nw) : 0;

    dim3 grid(p.NB, (unsigned)ceil_div(p.T, 16 * tb));
    if (is_f32) {
        switch (mode) {
        case kModeMglu: return launch_nmp<F32Traits, kModeMglu>(p, nmp, tb, nw, lds, grid, stream);
        case kModeProjections: return launch_nmp<F32Traits, kModeProjections>(p, nmp, tb, nw, lds, grid, stream);
        default: return launch_tb<F32Traits, 1, kModeSwiglu>(p, tb, nw, lds, grid, stream);
        }
    }
    switch (mode) {
    case kModeMglu: return launch_nmp<Bf16Traits, kModeMglu>(p, nmp, tb, nw, lds, grid, stream);
    case kModeProjections: return launch_nmp<Bf16Traits, kModeProjections>(p, nmp, tb, nw, lds, grid, stream);
    default: return launch_tb<Bf16Traits, 1, kModeSwiglu>(p, tb, nw, lds, grid, stream);
    }
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
