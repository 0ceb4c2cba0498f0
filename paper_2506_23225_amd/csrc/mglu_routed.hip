// Top-K routed MGLU at decode, reading only the selected masks.
//
// Paper: appendix "Top-K Routing": MGLU_TopK(x) = sum_i G(x)_i g(x (M_i*W)) * x ((1-M_i)*W) with G(x)
// non-zero for the K masks of largest router logit; only those K masked projections need be
// evaluated, which saves memory traffic as well as arithmetic.  Here that saving is taken on both
// sides: the masks come in the planar format (one contiguous run of words per column block and mask),
// the kernel finds which masks any token of its block selected, and streams W plus the planes of those
// masks only -- accumulators, operand preparation, MFMAs and mask bytes of every other mask are skipped.
//
// Structure = the resident streaming kernel (mglu_stream_impl.hpp): workgroup = one 16-column block,
// its wavefronts split K, x of the (at most 16) tokens sits in LDS in B-operand order, a ring of two
// register buffers per wavefront, sums combined in a fixed order through LDS, fused epilogue.  The
// kernel is compiled for NACT = 2, 4, 8 or 16 selected masks (their accumulators live in registers);
// the launcher picks NACT from the caller's k.  Should more masks be selected than NACT, the kernel
// makes another pass over W for the next NACT of them, so the result is right for any weights.
#include "mglu_stream_impl.hpp"

namespace mglu {

// The masked sums of one tile for the selected masks A, A + 1, ... (two per step: one 64-bit shift serves a pair).
// Written as a compile-time recursion so that every accumulator index is a constant whatever the unroller decides.
template <typename Tr, int NACT, int A>
__device__ __forceinline__ void routed_pairs(f32x4 (&acc)[1 + NACT], typename Tr::frag w, const uint32_t (&m)[NACT], int t,
                                             typename Tr::frag xf, int n_act)
{
    if constexpr (A < NACT) {
        if (A < n_act) {   // uniform over the workgroup
            typename Tr::frag fa, fb;
            Tr::flip_planar2(w, m[A], m[A + 1], t, fa, fb);
            acc[1 + A] = Tr::mma(fa, xf, acc[1 + A]);
            if (A + 1 < n_act) acc[2 + A] = Tr::mma(fb, xf, acc[2 + A]);
            routed_pairs<Tr, NACT, A + 2>(acc, w, m, t, xf, n_act);
        }
    }
}

template <typename Tr, int NACT>
struct RoutedChunk {
    typename Tr::frag w[Tr::TILES];
    uint32_t m[NACT];
};

// Wavefronts per SIMD the register allocation must leave room for (as in the resident kernel: told so,
// the compiler keeps the accumulators in ordinary registers and does not trade occupancy for scheduling freedom).
__host__ __device__ constexpr int routed_min_waves(int elem_bytes, int nact)
{
    return elem_bytes != 2 ? 2 : nact <= 2 ? 4 : nact <= 8 ? 3 : 2;
}

template <typename Tr, int NACT, int R>
__global__ __launch_bounds__(MGLU_STREAM_MAX_WAVES *kWave) __attribute__((amdgpu_waves_per_eu(routed_min_waves(Tr::ELEM_BYTES, NACT))))
void stream_routed_kernel(RoutedParams p, int nw_shift)
{
    constexpr int SETS = 1 + NACT;
    constexpr long CHUNK_BYTES = (long)kColBlock * kChunkK * Tr::ELEM_BYTES;
    typedef typename Tr::frag frag;
    typedef RoutedChunk<Tr, NACT> chunk_t;
    extern __shared__ f32x4 lds[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = 1 << nw_shift;
    const int r = lane & 15, q = lane >> 4;
    const int jb = blockIdx.x;
    const int tok0 = blockIdx.y * 16;
    const int tc = min(p.T - tok0, 16);

    const char *wbase = static_cast<const char *>(p.w) + (long)jb * p.NC * CHUNK_BYTES + lane * 16;
    // planar masks of this column block (uniform over the workgroup); plane i, chunk kc, lane l: + ((i NC + kc) 64 + l) words
    const char *mblock = reinterpret_cast<const char *>(p.m) + (long)jb * p.n_masks * p.NC * (kWave * 4);
    const uint32_t lane4 = lane * 4;

    frag *lds_x = reinterpret_cast<frag *>(lds);
    const int tsh = resident_row_shift(tc);
    const int x_frags = (p.NC * Tr::TILES * 4) << tsh;
    f32x4 *lds_red = lds + resident_x_frags_padded(x_frags, nw_shift);

    // ---- Start-up, ordered so that nothing waits for more than it needs (loads complete in issue order): the
    //      route weights first (a few words from L2), then the first R chunks of W (they do not depend on the
    //      routing), then -- once the weights are there, W still in flight -- the selection and the selected
    //      masks' words of those chunks, and last the copy of x into LDS. ----
    const int n_my = (p.NC - wave + nw - 1) >> nw_shift;   // chunks this wavefront owns (NC >= nw)
    auto kc_of = [&](int i) __attribute__((always_inline)) { return wave + i * nw; };
    const float *my_route = p.route + (long)(tok0 + min(r, tc - 1)) * p.n_masks;   // lane (r, q) holds token tok0 + r
    float w_all[kMaxMasks];
#pragma unroll
    for (int i = 0; i < kMaxMasks; ++i) w_all[i] = my_route[min(i, p.n_masks - 1)];
    auto load_w = [&](chunk_t &c, int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < Tr::TILES; ++t)
            c.w[t] = stream_load(reinterpret_cast<const frag *>(wbase + (long)kc * CHUNK_BYTES + t * 1024));
    };
    chunk_t buf[R];
#pragma unroll
    for (int s = 0; s < R; ++s) load_w(buf[s], kc_of(min(s, n_my - 1)));

    // which masks did any token of this block select?
    uint32_t active = 0u;
#pragma unroll
    for (int i = 0; i < kMaxMasks; ++i)
        if (__builtin_amdgcn_ballot_w64(i < p.n_masks && r < tc && w_all[i] != 0.0f) != 0) active |= 1u << i;
    active = __builtin_amdgcn_readfirstlane(active);   // the same in every wavefront: all read the same weights
    const int total = __builtin_popcount(active);

    // the first NACT selected masks in compact order; slots past the last selected mask repeat it (their loads
    // stay in bounds, their sums are never formed); with nothing selected everything points at mask 0
    const EpilogueParams ep = {p.n_masks, p.gate_fn, 0, p.route, p.n_masks};
    const uint32_t plane_bytes = (uint32_t)p.NC * (kWave * 4);
    const int n_act = min(NACT, total);
    uint32_t poff[NACT];   // byte offset of each selected mask's plane inside the column block (uniform)
    float rw[NACT];        // this lane's token's weight for it
    {
        uint32_t rest = active;
        int last = 0;
#pragma unroll
        for (int a = 0; a < NACT; ++a) {
            const int i = rest ? __builtin_ctz(rest) : last;
            last = i;
            rest &= rest - 1;
            poff[a] = (uint32_t)i * plane_bytes;
            rw[a] = w_all[0];
#pragma unroll
            for (int m = 1; m < kMaxMasks; ++m) rw[a] = i == m ? w_all[m] : rw[a];
            if (a >= n_act) rw[a] = 0.0f;
        }
    }
    auto load_m = [&](chunk_t &c, int kc) __attribute__((always_inline)) {
#pragma unroll
        for (int a = 0; a < NACT; ++a)
            c.m[a] = stream_load(reinterpret_cast<const uint32_t *>(mblock + (poff[a] + (uint32_t)kc * (kWave * 4)) + lane4));
    };
    auto load_chunk = [&](chunk_t &c, int kc) __attribute__((always_inline)) {
        load_w(c, kc);
        load_m(c, kc);
    };
#pragma unroll
    for (int s = 0; s < R; ++s) load_m(buf[s], kc_of(min(s, n_my - 1)));

    // x of this token block into LDS, fragment order: f = (g << tsh) + row holds x[tok0 + row][g LANE_K ..)
    for (int f = threadIdx.x; f < x_frags; f += nw * kWave) {
        const int row = min(f & ((1 << tsh) - 1), tc - 1), g = f >> tsh;
        const long k0 = min((long)g * Tr::LANE_K, (long)p.h - Tr::LANE_K);
        frag v = *reinterpret_cast<const frag *>(static_cast<const char *>(p.x) + ((long)(tok0 + row) * p.h + k0) * Tr::ELEM_BYTES);
        if (g * Tr::LANE_K >= p.h) v = frag{0, 0, 0, 0};
        lds_x[f] = v;
    }
    __syncthreads();

    f32x4 y = {0.f, 0.f, 0.f, 0.f};   // wavefront 0: the output
    f32x4 t_sum = {0.f, 0.f, 0.f, 0.f};   // wavefront 0: the reduced unmasked sum, kept for the masks beyond NACT

    if (total > 0) {
        // ---- main pass: W and the first NACT selected masks ----
        f32x4 acc[SETS];
#pragma unroll
        for (int s = 0; s < SETS; ++s) acc[s] = f32x4{0.f, 0.f, 0.f, 0.f};

        auto compute = [&](const chunk_t &c, int kc) __attribute__((always_inline)) {
#pragma unroll
            for (int t = 0; t < Tr::TILES; ++t) {
                frag xf = frag{0, 0, 0, 0};
                if (r < tc) xf = lds_x[((((kc * Tr::TILES + t) * 4 + q)) << tsh) + r];
                acc[0] = Tr::mma(c.w[t], xf, acc[0]);
                routed_pairs<Tr, NACT, 0>(acc, c.w[t], c.m, t, xf, n_act);
            }
        };

        // ring of R register buffers, as in the resident kernel (filled above): every load is unconditional
        int i0 = 0;
        for (; i0 + 2 * R <= n_my; i0 += R) {
#pragma unroll
            for (int s = 0; s < R; ++s) {
                compute(buf[s], kc_of(i0 + s));
                load_chunk(buf[s], kc_of(i0 + R + s));
            }
        }
#pragma unroll
        for (int s = 0; s < R; ++s) {
            if (i0 + s >= n_my) break;
            compute(buf[s], kc_of(i0 + s));
            if (i0 + R + s < n_my) load_chunk(buf[s], kc_of(i0 + R + s));
        }
#pragma unroll
        for (int s = 0; s < R; ++s) {
            if (i0 + R + s >= n_my) break;
            compute(buf[s], kc_of(i0 + R + s));
        }

        // combine the K split in wavefront order (fixed order => reproducible bits), then the terms of Eq. 3
        if (nw > 1) {
            if (wave > 0 && r < tc) {
#pragma unroll
                for (int s = 0; s < SETS; ++s) lds_red[((wave - 1) * SETS + s) * (4 * tc) + q * tc + r] = acc[s];
            }
            __syncthreads();
            if (wave == 0 && r < tc) {
                for (int w = 1; w < nw; ++w)
#pragma unroll
                    for (int s = 0; s < SETS; ++s) acc[s] += lds_red[((w - 1) * SETS + s) * (4 * tc) + q * tc + r];
            }
        }
        if (wave == 0) {
            t_sum = acc[0];
#pragma unroll
            for (int a = 0; a < NACT; ++a) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (a < n_act) y[c] += rw[a] * mglu_term(ep, acc[0][c], acc[1 + a][c]);
            }
        }
    }

    // ---- safety net: more masks selected than the kernel was sized for (the caller's k was too small).
    //      Two more masks per pass over W, one chunk at a time, nothing kept in flight: slow, but the
    //      result stays right for any weights. ----
    for (int base = NACT; base < total; base += 2) {
        uint32_t rest = active;
        for (int s = 0; s < base; ++s) rest &= rest - 1;
        const int i_a = __builtin_ctz(rest);
        rest &= rest - 1;
        const bool two = rest != 0;
        const int i_b = two ? __builtin_ctz(rest) : i_a;
        const float rw_a = my_route[i_a], rw_b = two ? my_route[i_b] : 0.0f;
        f32x4 ea = {0.f, 0.f, 0.f, 0.f}, eb = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
        for (int i = 0; i < n_my; ++i) {
            const int kc = kc_of(i);
#pragma unroll 1
            for (int t = 0; t < Tr::TILES; ++t) {
                const frag wf = *reinterpret_cast<const frag *>(wbase + (long)kc * CHUNK_BYTES + t * 1024);
                const uint32_t ma = *reinterpret_cast<const uint32_t *>(mblock + ((uint32_t)i_a * plane_bytes + (uint32_t)kc * (kWave * 4)) + lane4);
                const uint32_t mb = *reinterpret_cast<const uint32_t *>(mblock + ((uint32_t)i_b * plane_bytes + (uint32_t)kc * (kWave * 4)) + lane4);
                frag xf = frag{0, 0, 0, 0};
                if (r < tc) xf = lds_x[((((kc * Tr::TILES + t) * 4 + q)) << tsh) + r];
                frag fa, fb;
                Tr::flip_planar2(wf, ma, mb, t, fa, fb);
                ea = Tr::mma(fa, xf, ea);
                eb = Tr::mma(fb, xf, eb);
            }
        }
        if (nw > 1) {
            __syncthreads();   // the hand-over area may still be read by wavefront 0
            if (wave > 0 && r < tc) {
                lds_red[((wave - 1) * 2 + 0) * (4 * tc) + q * tc + r] = ea;
                lds_red[((wave - 1) * 2 + 1) * (4 * tc) + q * tc + r] = eb;
            }
            __syncthreads();
            if (wave == 0 && r < tc) {
                for (int w = 1; w < nw; ++w) {
                    ea += lds_red[((w - 1) * 2 + 0) * (4 * tc) + q * tc + r];
                    eb += lds_red[((w - 1) * 2 + 1) * (4 * tc) + q * tc + r];
                }
            }
        }
        if (wave == 0) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                y[c] += rw_a * mglu_term(ep, t_sum[c], ea[c]);
                if (two) y[c] += rw_b * mglu_term(ep, t_sum[c], eb[c]);
            }
        }
    }

    const int j0 = jb * kColBlock + 4 * q;
    if (wave == 0 && r < tc && j0 < p.d) {
        const long o = (long)(tok0 + r) * p.d + j0;
        if ((j0 + 3 < p.d) && ((p.d & 3) == 0)) {
            Tr::store4(p.out, o, y);
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (j0 + c < p.d) Tr::store1(p.out, o + c, y[c]);
        }
    }
}

// ---- host side --------------------------------------------------------------------------------

static int routed_nact(const RoutedParams &p)
{
    const long want = (long)p.k * (p.T < 16 ? p.T : 16);
    const int n = (int)(want < p.n_masks ? want : p.n_masks);
    return n <= 2 ? 2 : n <= 4 ? 4 : n <= 8 ? 8 : 16;
}

static StreamPlan routed_plan(const RoutedParams &p, int elem)
{
    StreamParams sp = {};
    sp.T = p.T; sp.h = p.h; sp.d = p.d; sp.NB = p.NB; sp.NC = p.NC; sp.n_masks = p.n_masks;
    const int nact = routed_nact(p);
    return plan_stream(sp, elem, nact, 1 + nact);
}

bool routed_supported(const RoutedParams &p, int elem) { return routed_plan(p, elem).resident; }

template <typename Tr, int NACT>
static hipError_t launch_routed_one(const RoutedParams &p, const StreamPlan &pl, hipStream_t stream)
{
    if (p.describe) {
        snprintf(p.describe, p.describe_len, "stream_routed_kernel<%s, %d, %d>", traits_name<Tr>(), NACT, MGLU_STREAM_RING);
        return hipSuccess;
    }
    hipLaunchKernelGGL((stream_routed_kernel<Tr, NACT, MGLU_STREAM_RING>), pl.grid, pl.block, pl.lds, stream, p, pl.nw_shift);
    return hipGetLastError();
}

template <typename Tr>
static hipError_t launch_routed_t(const RoutedParams &p, int elem, hipStream_t stream)
{
    const StreamPlan pl = routed_plan(p, elem);
    if (!pl.resident) return hipErrorInvalidValue;
    switch (routed_nact(p)) {
    case 2: return launch_routed_one<Tr, 2>(p, pl, stream);
    case 4: return launch_routed_one<Tr, 4>(p, pl, stream);
    case 8: return launch_routed_one<Tr, 8>(p, pl, stream);
    default: return launch_routed_one<Tr, 16>(p, pl, stream);
    }
}

hipError_t launch_routed(const RoutedParams &p, int elem, hipStream_t stream)
{
    if (elem == kElemF32) return launch_routed_t<F32Traits>(p, elem, stream);
    if (elem == kElemF16) return launch_routed_t<F16Traits>(p, elem, stream);
    return launch_routed_t<Bf16Traits>(p, elem, stream);
}

}  // namespace mglu
