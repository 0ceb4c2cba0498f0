// Streaming MGLU kernels for decode and small batches (tokens <= 64): HBM-bound.
//
// Paper: section "FlashMGLU", Alg. 1 (split-K matrix-vector product with packed
// masks).  Kept from it: W and the packed mask words are read once, the unmasked
// sum and one sum per mask are accumulated together in registers, the value
// branch comes from the complement, partial sums of a K split are combined on
// chip.  Different from it, for gfx950:
//   - the multiply-accumulates run on the matrix cores (v_mfma_f32_16x16x32_bf16 / _f16,
//     four v_mfma_f32_16x16x4_f32 for fp32; tokens padded to 16 per tile), so the vector ALUs
//     only prepare operands;
//   - a mask bit flips the sign of its weight element (one shift + one 3-input
//     bit-op per register pair and mask) instead of predicating an add; the gate
//     and value sums are recovered as (t -/+ dsum)/2;
//   - the K split is across the wavefronts of one workgroup and is combined in a
//     fixed order through LDS -- no float atomics, bit-reproducible results;
//   - Swish, the gate*value products and the sum over masks are applied to the
//     reduced sums in registers and only `out` is written (Eq. 3).
//
// Two kernels share the chunk loader, the tile multiply and the epilogue:
//   stream_resident_kernel  up to 16 tokens whose rows of x fit in LDS: x is copied there
//                           once, in B-operand order; no barrier inside the K loop.
//   stream_panel_kernel     any token count up to 64: a workgroup owns NWC column blocks, its
//                           wavefronts (NWC x NWK) share panels of x (NWK chunks of K) staged
//                           through double-buffered LDS, one barrier per panel, so x is
//                           fetched once per NWC * 16 columns instead of once per 16.
// In both, a wavefront's chunks of one column block are interleaved with those of the other
// wavefronts that split K with it, so together they read one contiguous run of the packed
// weight stream at any moment.
#pragma once
#include <stdio.h>

#include <type_traits>

#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

// Tuning knobs (compile-time; the defaults are the measured best on MI355X).
#ifndef MGLU_STREAM_MAX_WAVES
#define MGLU_STREAM_MAX_WAVES 4   // resident kernel: wavefronts per workgroup = K-split ways
#endif
#ifndef MGLU_STREAM_RING
#define MGLU_STREAM_RING 2        // resident kernel: chunks of W a wavefront keeps in flight
#endif
#ifndef MGLU_RESIDENT_MAX_T
#define MGLU_RESIDENT_MAX_T 16    // most tokens the resident kernel takes (the panel kernel takes the rest)
#endif
// Resident kernel, main form only: launches with at most this many chunks of W per CU run a flavour
// that reads x from LDS in every lane (rows past T repeat the last one) instead of predicated.  The
// compiler then fetches the fragments further ahead: measured 2-3 % faster on the 2048 x 5632 shape
// (22 chunks per CU), 3-5 % slower from 4096 x 14336 (112 per CU) on.
#ifndef MGLU_RESIDENT_RX_MAX_CHUNKS_PER_CU
#define MGLU_RESIDENT_RX_MAX_CHUNKS_PER_CU 48
#endif
#ifndef MGLU_RESIDENT_FLOOR
#define MGLU_RESIDENT_FLOOR 1     // resident kernel: tell the register allocator how many wavefronts per SIMD to keep
#endif
#ifndef MGLU_RESIDENT_XPREFETCH
#define MGLU_RESIDENT_XPREFETCH 1   // resident kernel: read x fragments from LDS one tile ahead, into registers zeroed once
#endif
#ifndef MGLU_STREAM_NONTEMPORAL
#define MGLU_STREAM_NONTEMPORAL 1 // W and the masks are read once per call: mark the loads streaming
#endif
// Panel kernel workgroup shapes (column blocks x K-split ways x chunks per wavefront per panel):
// "wide" shares each x panel among 8 column blocks and needs d_ff / 128 workgroups to fill the
// chip; "split" halves the columns and splits K instead, for narrower layers.
#ifndef MGLU_PANEL_WIDE_MIN_WGS
#define MGLU_PANEL_WIDE_MIN_WGS 200
#endif

// Register budget of the panel kernel: always at least 2 wavefronts per SIMD (256 registers);
// instantiations with many accumulators (more than 12 sets x token blocks) are told to aim
// for exactly 2, or the compiler spills them down to 128 registers in pursuit of occupancy.
#define MGLU_PANEL_OCCUPANCY(SETS_X_TB) __attribute__((amdgpu_waves_per_eu(2, (SETS_X_TB) > 12 ? 2 : 8)))

namespace mglu {

// Resident kernel: x fragments each thread copies per group (a power of two), and the LDS x area
// rounded up to whole groups of the workgroup's 64 << nw_shift threads (so that every copy is
// unconditional).  Shifts only: this runs at the start of every workgroup.
constexpr int kResidentXGroupShift = 2;
constexpr int kResidentXGroup = 1 << kResidentXGroupShift;
// log2 of the rows per fragment group in the LDS copy of x: the token count rounded up to a power of two
__host__ __device__ constexpr int resident_row_shift(int tc) { return tc <= 1 ? 0 : tc <= 2 ? 1 : tc <= 4 ? 2 : tc <= 8 ? 3 : 4; }
__host__ __device__ constexpr int resident_x_frags_padded(int x_frags, int nw_shift)
{
    const int sh = kResidentXGroupShift + nw_shift + 6;
    return ((x_frags + (1 << sh) - 1) >> sh) << sh;
}

template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
#if MGLU_STREAM_NONTEMPORAL
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// Registers of one chunk in flight: W (or the two SwiGLU matrices) and the mask words.
template <typename Tr, int NMP, int MODE>
struct WChunk {
    typename Tr::frag w[Tr::TILES];
    typename Tr::frag w2[MODE == kModeSwiglu ? Tr::TILES : 1];
    uint32_t m[NMP];
};

// wp / wp2 / mp already point at this lane's place in the chunk.
template <typename Tr, int NMP, int MODE>
__device__ __forceinline__ void load_wchunk(WChunk<Tr, NMP, MODE> &c, const char *wp, const char *wp2, const uint32_t *mp)
{
    typedef typename Tr::frag frag;
#pragma unroll
    for (int t = 0; t < Tr::TILES; ++t) c.w[t] = stream_load(reinterpret_cast<const frag *>(wp + t * 1024));
    if constexpr (MODE == kModeSwiglu) {
#pragma unroll
        for (int t = 0; t < Tr::TILES; ++t) c.w2[t] = stream_load(reinterpret_cast<const frag *>(wp2 + t * 1024));
    } else if constexpr (MODE == kModeLinear) {
        (void)mp;
    } else if constexpr (NMP >= 8) {
#pragma unroll
        for (int piece = 0; piece < NMP / 4; ++piece) {
            u32x4 a = stream_load(reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(mp) + piece * kMaskPieceBytes));
#pragma unroll
            for (int i = 0; i < 4; ++i) c.m[4 * piece + i] = a[i];
        }
    } else if constexpr (NMP == 4) {
        u32x4 a = stream_load(reinterpret_cast<const u32x4 *>(mp));
#pragma unroll
        for (int i = 0; i < 4; ++i) c.m[i] = a[i];
    } else if constexpr (NMP == 2) {
        u32x2 a = stream_load(reinterpret_cast<const u32x2 *>(mp));
        c.m[0] = a.x; c.m[1] = a.y;
    } else {
        c.m[0] = stream_load(mp);
    }
}

// One 32-k (bf16) / 16-k (fp32) tile: t += W x, dsum_i += flip_i(W) x for every token block.
template <typename Tr, int NMP, int TB, int MODE>
__device__ __forceinline__ void mma_tile(f32x4 (&acc)[sets_of(MODE, NMP)][TB], const WChunk<Tr, NMP, MODE> &c, int t,
                                const typename Tr::frag (&xf)[TB])
{
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[0][tb] = Tr::mma(c.w[t], xf[tb], acc[0][tb]);
    if constexpr (MODE == kModeSwiglu) {
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[1][tb] = Tr::mma(c.w2[t], xf[tb], acc[1][tb]);
    } else if constexpr (MODE != kModeLinear) {
        // The flipped fragment of mask i + 1 is prepared in a second set of registers while the
        // MFMAs of mask i run, so the vector ALU and the matrix pipe work at the same time.
        typename Tr::frag wf[2];
        wf[0] = Tr::template flip<NMP>(c.w[t], c.m, t, 0);
#pragma unroll
        for (int i = 0; i < NMP; ++i) {
            if (i + 1 < NMP) wf[(i + 1) & 1] = Tr::template flip<NMP>(c.w[t], c.m, t, i + 1);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) acc[1 + i][tb] = Tr::mma(wf[i & 1], xf[tb], acc[1 + i][tb]);
        }
    }
}

// Epilogue on the reduced sums (Eq. 3): lane (r, q) holds token 16 tb + r, columns 4q .. 4q+3 of block jb.
// In the plain mode the mask count is the padded one, a compile-time constant: a padding mask is
// all-value (its packed words are zero), so its sum equals t bit for bit, its gate is exactly 0 and
// its term swish(0) * value = 0 -- computing it costs less than a run-time bound on every element.
template <int MODE, int NMP>
__device__ __forceinline__ EpilogueParams epilogue_params(const StreamParams &p)
{
    return MODE == kModeMgluVariant ? EpilogueParams{p.n_masks, p.gate_fn, p.mask_use, p.route, p.n_masks}
                                    : EpilogueParams{NMP, 0, 0, nullptr, 0};
}

// Four consecutive outputs of one token, rounded once to the output type; the last columns of a ragged d_ff one by one.
template <typename Tr>
__device__ __forceinline__ void store_out4(const StreamParams &p, f32x4 y, long o, int j0, bool full)
{
    if (full) {
        Tr::store4(p.out, o, y);
    } else {
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (j0 + c < p.d) Tr::store1(p.out, o + c, y[c]);
    }
}

// rw: the route weights of this lane's token of every token block (see route_weights).
template <typename Tr, int NMP, int TB, int MODE>
__device__ __forceinline__ void epilogue(const StreamParams &p, const f32x4 (&acc)[sets_of(MODE, NMP)][TB],
                                const float (&rw)[TB][NMP], int jb, int tok0, int r, int q)
{
    const int j0 = jb * kColBlock + 4 * q;
    if (j0 >= p.d) return;
    const bool full = (j0 + 3 < p.d) && ((p.d & 3) == 0);
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) {
        const long tok = (long)tok0 + 16 * tb + r;
        if (tok >= p.T) continue;
        const long o = tok * p.d + j0;
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
            const EpilogueParams ep = epilogue_params<MODE, NMP>(p);
            f32x4 y;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if constexpr (MODE == kModeSwiglu) {
                    y[c] = swish(acc[0][tb][c]) * acc[1][tb][c];
                } else if constexpr (MODE == kModeLinear) {
                    y[c] = acc[0][tb][c];
                } else {
                    float ds[NMP];
#pragma unroll
                    for (int i = 0; i < NMP; ++i) ds[i] = acc[1 + i][tb][c];
                    y[c] = mglu_mix<NMP, MODE == kModeMglu>(ep, rw[tb], acc[0][tb][c], ds);
                }
            }
            store_out4<Tr>(p, y, o, j0, full);
        }
    }
}

// ================================================================================================
// Resident kernel: workgroup (jb, tg) owns columns [16 jb, 16 jb + 16) for the token block tg of
// up to 16 tokens; its nw wavefronts take chunks kc = wave, wave + nw, ...
// ================================================================================================
// The arguments are passed one by one, the ones the first loads depend on first: the leading
// ones are delivered in scalar registers when the wavefront starts (kernel-argument preload,
// switched on in the build flags), which takes one memory round trip off the start of every
// workgroup.
// Wavefronts per SIMD the register allocation must leave room for.  Told so, the compiler keeps the
// accumulators of the 16-bit MGLU instantiations in ordinary registers and needs fewer in total
// (8 masks: 120 instead of 88 + 72 accumulator registers), without spilling.
__host__ __device__ constexpr int resident_min_waves(int elem_bytes, int mode, int nmp)
{
    if (!MGLU_RESIDENT_FLOOR || elem_bytes != 2 || mode == kModeSwiglu || mode == kModeLinear) return 1;
    return nmp <= 1 ? 5 : nmp <= 4 ? 4 : nmp <= 8 ? 3 : 2;
}

template <typename Tr, int NMP, int MODE, int R, bool RX>
__global__ __launch_bounds__(MGLU_STREAM_MAX_WAVES *kWave)
__attribute__((amdgpu_waves_per_eu(resident_min_waves(Tr::ELEM_BYTES, MODE, NMP)))) void stream_resident_kernel(
    const void *a_w, const uint32_t *a_m, const void *a_x, int a_NC, int a_T, int a_h, int a_d, void *a_out,
    int a_nw_shift, int a_n_masks, int a_NB, const void *a_w2, float *a_proj_t, float *a_proj_gate, float *a_proj_value,
    int a_gate_fn, int a_mask_use, const float *a_route)
{
    StreamParams p;
    p.x = a_x; p.w = a_w; p.w2 = a_w2; p.m = a_m; p.out = a_out;
    p.proj_t = a_proj_t; p.proj_gate = a_proj_gate; p.proj_value = a_proj_value;
    p.T = a_T; p.h = a_h; p.d = a_d; p.n_masks = a_n_masks; p.NB = a_NB; p.NC = a_NC;
    p.gate_fn = a_gate_fn; p.mask_use = a_mask_use; p.route = a_route;
    constexpr int SETS = sets_of(MODE, NMP);
    constexpr long CHUNK_BYTES = (long)kColBlock * kChunkK * Tr::ELEM_BYTES;
    typedef typename Tr::frag frag;
    typedef WChunk<Tr, NMP, MODE> chunk_t;
    extern __shared__ f32x4 lds[];

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int nw = 1 << a_nw_shift;      // wavefronts of this workgroup (= blockDim.x / 64), a power of two
    const int r = lane & 15, q = lane >> 4;
    const int jb = blockIdx.x;
    const int tok0 = blockIdx.y * 16;
    const int tc = min(p.T - tok0, 16);  // token lanes that carry data

    const char *wbase = static_cast<const char *>(p.w) + (long)jb * p.NC * CHUNK_BYTES + lane * 16;
    const char *w2base = static_cast<const char *>(p.w2) + (long)jb * p.NC * CHUNK_BYTES + lane * 16;
    const uint32_t *mbase = reinterpret_cast<const uint32_t *>(
        reinterpret_cast<const char *>(p.m + (long)jb * p.NC * kWave * NMP) + mask_lane_bytes<NMP>(lane));

    // LDS: [x fragments of this token block][hand-over area of the K-split reduction].  A fragment
    // group g (LANE_K consecutive k) holds 2^tsh >= tc rows, so positions split with shifts only.
    frag *lds_x = reinterpret_cast<frag *>(lds);
    const int tsh = resident_row_shift(tc);
    const int x_frags = (p.NC * Tr::TILES * 4) << tsh;
    f32x4 *lds_red = lds + resident_x_frags_padded(x_frags, a_nw_shift);

    f32x4 acc[SETS][1];
#pragma unroll
    for (int s = 0; s < SETS; ++s) acc[s][0] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Routed layer (appendix "Top-K Routing"): a mask that no token of this block selected needs no
    // sum at all.  The selected masks idx[0 .. n_act) take the accumulator sets 1 .. n_act, and the
    // route weights follow them; everything here is uniform over the workgroup.
    float rw[1][NMP];
    int n_act = p.n_masks;
    int idx[NMP];
#pragma unroll
    for (int i = 0; i < NMP; ++i) idx[i] = i;
    if constexpr (MODE == kModeMgluVariant) {
        float w_all[NMP];
        route_weights<NMP>(epilogue_params<MODE, NMP>(p), tok0 + r, r < tc, w_all);
        uint32_t active = 0u;
#pragma unroll
        for (int i = 0; i < NMP; ++i)
            if (i < p.n_masks && __builtin_amdgcn_ballot_w64(r < tc && w_all[i] != 0.0f) != 0) active |= 1u << i;
        n_act = __builtin_popcount(active);
#pragma unroll
        for (int a = 0; a < NMP; ++a) {
            idx[a] = active ? __builtin_ctz(active) : 0;
            active &= active - 1;
            rw[0][a] = w_all[0];
#pragma unroll
            for (int i = 1; i < NMP; ++i) rw[0][a] = idx[a] == i ? w_all[i] : rw[0][a];
        }
        p.n_masks = n_act;  // what the epilogue sums over
    } else {
        route_weights<NMP>(epilogue_params<MODE, NMP>(p), tok0 + r, false, rw[0]);
    }
    // the weights of the masks this wavefront finishes in the shared epilogue: (compact) index wave + a * nw
    float rw_mine[NMP];
#pragma unroll
    for (int a = 0; a < NMP; ++a) {
        rw_mine[a] = rw[0][0];
#pragma unroll
        for (int i = 1; i < NMP; ++i) rw_mine[a] = (wave + a * nw == i) ? rw[0][i] : rw_mine[a];
    }

    auto load_chunk = [&](chunk_t &c, int kc) __attribute__((always_inline)) {
        load_wchunk<Tr, NMP, MODE>(c, wbase + (long)kc * CHUNK_BYTES, w2base + (long)kc * CHUNK_BYTES,
                                   mbase + (long)kc * kWave * NMP);
    };
    // B-operand lanes past the last token: zero (predicated read), or in the RX flavour the last
    // token's row again; either way their accumulator columns are never stored
    const int rx = RX ? min(r, tc - 1) : r;
    const int n_my = (p.NC - wave + nw - 1) >> a_nw_shift;  // chunks this wavefront owns (NC >= nw, so >= 1)
    auto kc_of = [&](int i) __attribute__((always_inline)) { return wave + i * nw; };
    frag xq[2] = {frag{0, 0, 0, 0}, frag{0, 0, 0, 0}};
    auto x_read = [&](frag &dst, int kc, int t) __attribute__((always_inline)) {
        if (RX || r < tc) dst = lds_x[((((kc * Tr::TILES + t) * 4 + q)) << tsh) + rx];
    };
    // multiply this wavefront's i-th chunk (held in c)
    auto compute = [&](const chunk_t &c, int i) __attribute__((always_inline)) {
        const int kc = kc_of(i);
        if constexpr (MODE == kModeMgluVariant) {
#pragma unroll
            for (int t = 0; t < Tr::TILES; ++t) {
                frag xf = frag{0, 0, 0, 0};
                if (RX || r < tc) xf = lds_x[((((kc * Tr::TILES + t) * 4 + q)) << tsh) + rx];
                acc[0][0] = Tr::mma(c.w[t], xf, acc[0][0]);
#pragma unroll
                for (int a = 0; a < NMP; ++a) {
                    if (a >= n_act) break;  // uniform
                    acc[1 + a][0] = Tr::mma(Tr::template flip_at<NMP>(c.w[t], c.m, t, idx[a]), xf, acc[1 + a][0]);
                }
            }
        } else if constexpr (MGLU_RESIDENT_XPREFETCH) {
            // x fragments are read from LDS one tile ahead of their use, in turn into two registers sets that were
            // zeroed once: the lanes past the last token are never written (predicated read), so they stay zero
            // without being cleared for every tile, and the LDS latency hides behind the tile before.
            const int kc_next = kc_of(min(i + 1, n_my - 1));
#pragma unroll
            for (int t = 0; t < Tr::TILES; ++t) {
                if (t + 1 < Tr::TILES) x_read(xq[(t + 1) & 1], kc, t + 1);
                else x_read(xq[0], kc_next, 0);
                const frag xf[1] = {xq[t & 1]};
                mma_tile<Tr, NMP, 1, MODE>(acc, c, t, xf);
            }
        } else {
#pragma unroll
            for (int t = 0; t < Tr::TILES; ++t) {
                frag xf[1] = {frag{0, 0, 0, 0}};
                if (RX || r < tc) xf[0] = lds_x[((((kc * Tr::TILES + t) * 4 + q)) << tsh) + rx];
                mma_tile<Tr, NMP, 1, MODE>(acc, c, t, xf);
            }
        }
    };

    // ---- A ring of R register buffers, indexed at compile time.  All R are loaded before anything
    //      else waits, so a wavefront that owns at most R chunks has its whole share of W in flight
    //      at once; otherwise a buffer is refilled right after it has been multiplied.  In the
    //      steady-state loop every load is unconditional, which lets the compiler wait for exactly
    //      the chunk it multiplies. ----
    chunk_t buf[R];
    {
        // Copy this token block's x into LDS in fragment order: fragment f = (g << tsh) + row holds
        // x[tok0 + row][g * LANE_K .. + LANE_K), zero beyond d_model (rows >= tc repeat the last row).  The first group of x loads
        // is issued before the W loads and, hitting L2, returns before them.  Loads and stores are
        // unconditional (indices clamped, the LDS area padded to whole groups): a load whose only
        // use sat under a condition would be moved behind the W loads and wait for all of them.
        const int nthr = nw * kWave;
        auto x_load = [&](int f) __attribute__((always_inline)) {
            const int fc = min(f, x_frags - 1);  // clamped: the load is always in bounds
            const int row = min(fc & ((1 << tsh) - 1), tc - 1), g = fc >> tsh;
            const long k0 = min((long)g * Tr::LANE_K, (long)p.h - Tr::LANE_K);
            return *reinterpret_cast<const frag *>(static_cast<const char *>(p.x) +
                                                   ((long)(tok0 + row) * p.h + k0) * Tr::ELEM_BYTES);
        };
        auto x_store = [&](int f, frag v) __attribute__((always_inline)) {
            if ((f >> tsh) * Tr::LANE_K >= p.h) v = frag{0, 0, 0, 0};
            lds_x[f] = v;
        };
        frag xv[kResidentXGroup];
#pragma unroll
        for (int b = 0; b < kResidentXGroup; ++b) xv[b] = x_load(threadIdx.x + b * nthr);
#pragma unroll
        for (int s = 0; s < R; ++s) load_chunk(buf[s], kc_of(min(s, n_my - 1)));
        __builtin_amdgcn_sched_barrier(0);  // every load above is issued before the first wait below
#pragma unroll
        for (int b = 0; b < kResidentXGroup; ++b) x_store(threadIdx.x + b * nthr, xv[b]);
        for (int f0 = threadIdx.x + kResidentXGroup * nthr; f0 < x_frags; f0 += kResidentXGroup * nthr) {
#pragma unroll
            for (int b = 0; b < kResidentXGroup; ++b) xv[b] = x_load(f0 + b * nthr);
#pragma unroll
            for (int b = 0; b < kResidentXGroup; ++b) x_store(f0 + b * nthr, xv[b]);
        }
        __syncthreads();
    }
    if constexpr (MGLU_RESIDENT_XPREFETCH && MODE != kModeMgluVariant) x_read(xq[0], kc_of(0), 0);

    int i0 = 0;
    for (; i0 + 2 * R <= n_my; i0 += R) {  // every buffer of the ring has a chunk left to refill it
#pragma unroll
        for (int s = 0; s < R; ++s) {
            compute(buf[s], i0 + s);
            load_chunk(buf[s], kc_of(i0 + R + s));
        }
    }
    // tail: chunks i0 .. n_my - 1, fewer than 2 R; those below i0 + R are in the ring already
#pragma unroll
    for (int s = 0; s < R; ++s) {
        if (i0 + s >= n_my) break;  // uniform over the wavefront
        compute(buf[s], i0 + s);
        if (i0 + R + s < n_my) load_chunk(buf[s], kc_of(i0 + R + s));
    }
#pragma unroll
    for (int s = 0; s < R; ++s) {
        if (i0 + R + s >= n_my) break;
        compute(buf[s], i0 + R + s);
    }

    // ---- combine the K split and finish.  Sums are always added in wavefront order (fixed order =>
    //      reproducible bits). ----
    if constexpr (MODE == kModeMglu || MODE == kModeMgluVariant) {
        if (nw > 1) {
            // Eq. 3 costs a few hundred instructions per lane (an exp, a reciprocal per column and
            // mask), which one wavefront at the end of every workgroup would run alone: every
            // wavefront publishes its sums, then wavefront w finishes the masks w, w + nw, ... and
            // wavefront 0 adds the shares.
            f32x4 *lds_term = lds_red + nw * SETS * 4 * tc;
            const int slot = q * tc + r;
            if (r < tc) {
#pragma unroll
                for (int s = 0; s < SETS; ++s) lds_red[(wave * SETS + s) * (4 * tc) + slot] = acc[s][0];
            }
            __syncthreads();
            if (r < tc) {
                const EpilogueParams ep = epilogue_params<MODE, NMP>(p);
                f32x4 t = lds_red[slot];
                for (int w = 1; w < nw; ++w) t += lds_red[(w * SETS) * (4 * tc) + slot];
                f32x4 share = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int a = 0; a < NMP; ++a) {
                    const int i = wave + a * nw;
                    if (i >= p.n_masks) break;  // uniform over the wavefront
                    f32x4 ds = lds_red[(1 + i) * (4 * tc) + slot];
                    for (int w = 1; w < nw; ++w) ds += lds_red[(w * SETS + 1 + i) * (4 * tc) + slot];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        const float term = mglu_term(ep, t[c], ds[c]);
                        share[c] += ep.route ? rw_mine[a] * term : term;
                    }
                }
                lds_term[wave * (4 * tc) + slot] = share;
            }
            __syncthreads();
            const int j0 = jb * kColBlock + 4 * q;
            if (wave == 0 && r < tc && j0 < p.d) {
                f32x4 y = lds_term[slot];
                for (int w = 1; w < nw; ++w) y += lds_term[w * (4 * tc) + slot];
                store_out4<Tr>(p, y, (long)(tok0 + r) * p.d + j0, j0, (j0 + 3 < p.d) && ((p.d & 3) == 0));
            }
        } else {
            epilogue<Tr, NMP, 1, MODE>(p, acc, rw, jb, tok0, r, q);
        }
    } else {
        // wavefronts 1..nw-1 hand their sums to wavefront 0 through LDS
        if (nw > 1) {
            if (wave > 0 && r < tc) {
#pragma unroll
                for (int s = 0; s < SETS; ++s) lds_red[((wave - 1) * SETS + s) * (4 * tc) + q * tc + r] = acc[s][0];
            }
            __syncthreads();
            if (wave == 0 && r < tc) {
                for (int w = 1; w < nw; ++w)
#pragma unroll
                    for (int s = 0; s < SETS; ++s) acc[s][0] += lds_red[((w - 1) * SETS + s) * (4 * tc) + q * tc + r];
            }
        }
        if (wave == 0) epilogue<Tr, NMP, 1, MODE>(p, acc, rw, jb, tok0, r, q);
    }
}

// ================================================================================================
// Panel kernel: workgroup (jg, tg) owns NWC column blocks for the token group tg of 16 * TB tokens.
// Wavefront (c, s) = (wave / NWK, wave % NWK) works on column block jg * NWC + c; its g-th chunk is
// kc = g * NWK + s.  A panel is NWK * CPW consecutive chunks of K (CPW chunks per wavefront); the x
// rows of a panel (all 16 * TB tokens) are staged once per workgroup into LDS in B-operand order,
// double-buffered: the loads for panel i + 1 are issued before panel i is multiplied and written
// to LDS after it, with one barrier per panel.
// ================================================================================================
template <typename Tr, int NMP, int TB, int MODE, int NWC, int NWK, int CPW>
__global__ __launch_bounds__(NWC *NWK *kWave) MGLU_PANEL_OCCUPANCY(sets_of(MODE, NMP) * TB)
void stream_panel_kernel(StreamParams p)
{
    constexpr int SETS = sets_of(MODE, NMP);
    constexpr int NW = NWC * NWK;
    constexpr long CHUNK_BYTES = (long)kColBlock * kChunkK * Tr::ELEM_BYTES;
    constexpr int CHUNK_FRAG_TILES = Tr::TILES * TB;               // 1 KiB fragment tiles of x per chunk
    constexpr int PANEL_FRAG_TILES = NWK * CPW * CHUNK_FRAG_TILES;
    constexpr int XF = PANEL_FRAG_TILES / NW;                      // fragment tiles each wavefront stages
    static_assert(PANEL_FRAG_TILES % NW == 0, "x panel must split evenly over the wavefronts");
    typedef typename Tr::frag frag;
    typedef WChunk<Tr, NMP, MODE> chunk_t;
    extern __shared__ f32x4 lds[];
    frag *lds_x = reinterpret_cast<frag *>(lds);                   // [2][PANEL_FRAG_TILES][64]

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int c = wave / NWK, s = wave % NWK;
    const int jb = blockIdx.x * NWC + c;
    const long jbc = min(jb, p.NB - 1);   // column blocks past the end: loads clamped, store dropped
    const int tok0 = blockIdx.y * (16 * TB);

    const char *wbase = static_cast<const char *>(p.w) + jbc * p.NC * CHUNK_BYTES + lane * 16;
    const char *w2base = static_cast<const char *>(p.w2) + jbc * p.NC * CHUNK_BYTES + lane * 16;
    const uint32_t *mbase = reinterpret_cast<const uint32_t *>(
        reinterpret_cast<const char *>(p.m + jbc * p.NC * kWave * NMP) + mask_lane_bytes<NMP>(lane));

    f32x4 acc[SETS][TB];
#pragma unroll
    for (int st = 0; st < SETS; ++st)
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) acc[st][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int n_panels = (p.NC + NWK * CPW - 1) / (NWK * CPW);
    auto load_chunk = [&](chunk_t &ck, int g) __attribute__((always_inline)) {
        const long kc = min(g * NWK + s, p.NC - 1);   // clamped: always in bounds
        load_wchunk<Tr, NMP, MODE>(ck, wbase + kc * CHUNK_BYTES, w2base + kc * CHUNK_BYTES, mbase + kc * kWave * NMP);
    };
    // fragment tile ft = (chunk-in-panel * TILES + t) * TB + tb; this wavefront stages ft = wave + NW i
    auto x_load = [&](int panel, int i) __attribute__((always_inline)) {
        const int ft = wave + NW * i;
        const int ch = ft / CHUNK_FRAG_TILES, t = (ft / TB) % Tr::TILES, tb = ft % TB;
        const long tok = min((long)tok0 + 16 * tb + r, (long)p.T - 1);
        const long k0 = min((long)(panel * NWK * CPW + ch) * kChunkK + t * Tr::TILE_K + q * Tr::LANE_K,
                            (long)p.h - Tr::LANE_K);
        return *reinterpret_cast<const frag *>(static_cast<const char *>(p.x) + (tok * p.h + k0) * Tr::ELEM_BYTES);
    };
    auto x_store = [&](int buf, int panel, int i, frag v) __attribute__((always_inline)) {
        const int ft = wave + NW * i;
        const int ch = ft / CHUNK_FRAG_TILES, t = (ft / TB) % Tr::TILES, tb = ft % TB;
        const bool ok = (tok0 + 16 * tb + r < p.T) &&
                        ((long)(panel * NWK * CPW + ch) * kChunkK + t * Tr::TILE_K + q * Tr::LANE_K < p.h);
        lds_x[(buf * PANEL_FRAG_TILES + ft) * kWave + lane] = ok ? v : frag{0, 0, 0, 0};
    };
    // multiply this wavefront's j-th chunk of a panel whose x sits in LDS buffer `buf`
    auto compute = [&](const chunk_t &ck, int buf, int panel, int j) __attribute__((always_inline)) {
        if ((panel * CPW + j) * NWK + s >= p.NC) return;   // no such chunk (tail of the last panel)
        const frag *xb = lds_x + (buf * PANEL_FRAG_TILES + (j * NWK + s) * CHUNK_FRAG_TILES) * kWave + lane;
#pragma unroll
        for (int t = 0; t < Tr::TILES; ++t) {
            frag xf[TB];
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) xf[tb] = xb[(t * TB + tb) * kWave];
            mma_tile<Tr, NMP, TB, MODE>(acc, ck, t, xf);
        }
    };

    chunk_t bufs[2];
    frag xv[XF];
    // prologue: x of panel 0 first (L2 hits return ahead of the W loads issued after them)
#pragma unroll
    for (int i = 0; i < XF; ++i) xv[i] = x_load(0, i);
    load_chunk(bufs[0], 0);
#pragma unroll
    for (int i = 0; i < XF; ++i) x_store(0, 0, i, xv[i]);
    __syncthreads();

    // One panel that has a successor: fetch the next panel's x, stream this panel's chunks (each
    // multiply overlapped with the next chunk's loads), publish the next x.  PAR = register-buffer
    // parity of the panel's first chunk and XB = its LDS buffer, both compile-time.
    auto panel_step = [&](int panel, auto par_tag, auto xb_tag) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value, XB = decltype(xb_tag)::value;
#pragma unroll
        for (int i = 0; i < XF; ++i) xv[i] = x_load(panel + 1, i);
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            load_chunk(bufs[(PAR + j + 1) & 1], panel * CPW + j + 1);
            compute(bufs[(PAR + j) & 1], XB, panel, j);
        }
#pragma unroll
        for (int i = 0; i < XF; ++i) x_store(XB ^ 1, panel + 1, i, xv[i]);
        __syncthreads();
    };
    // The last panel: nothing left to stage, and no load after the final chunk.
    auto last_panel = [&](int panel, auto par_tag, auto xb_tag) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_tag)::value, XB = decltype(xb_tag)::value;
#pragma unroll
        for (int j = 0; j < CPW; ++j) {
            if (j + 1 < CPW) load_chunk(bufs[(PAR + j + 1) & 1], panel * CPW + j + 1);
            compute(bufs[(PAR + j) & 1], XB, panel, j);
        }
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    constexpr int PAR1 = CPW & 1;   // parity of the first chunk of an odd panel
    int pn = 0;
    for (; pn + 2 < n_panels; pn += 2) {
        panel_step(pn, I0{}, I0{});
        panel_step(pn + 1, std::integral_constant<int, PAR1>{}, I1{});
    }
    if (n_panels - pn == 2) {
        panel_step(pn, I0{}, I0{});
        last_panel(pn + 1, std::integral_constant<int, PAR1>{}, I1{});
    } else {
        last_panel(pn, I0{}, I0{});
    }

    // ---- combine the K split per column block: wavefronts s > 0 hand their sums to (c, 0) through
    //      LDS (the x buffers are free now), added in order of s ----
    if constexpr (NWK > 1) {
        __syncthreads();
        if (s > 0) {
#pragma unroll
            for (int st = 0; st < SETS; ++st)
#pragma unroll
                for (int tb = 0; tb < TB; ++tb)
                    lds[(((c * (NWK - 1) + s - 1) * SETS + st) * TB + tb) * kWave + lane] = acc[st][tb];
        }
        __syncthreads();
        if (s == 0) {
#pragma unroll
            for (int w = 1; w < NWK; ++w)
#pragma unroll
                for (int st = 0; st < SETS; ++st)
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
                        acc[st][tb] += lds[(((c * (NWK - 1) + w - 1) * SETS + st) * TB + tb) * kWave + lane];
        }
    }
    if (s == 0 && jb < p.NB) {
        // route weights: read here, not ahead of the K loop (this kernel has no registers to hold them
        // across it, and its workgroups run long enough that the read's latency does not show)
        float rw[TB][NMP];
#pragma unroll
        for (int tb = 0; tb < TB; ++tb)
            route_weights<NMP>(epilogue_params<MODE, NMP>(p), tok0 + 16 * tb + r, tok0 + 16 * tb + r < p.T, rw[tb]);
        epilogue<Tr, NMP, TB, MODE>(p, acc, rw, jb, tok0, r, q);
    }
}

// ---- host side --------------------------------------------------------------------------------


struct PanelWide  { static constexpr int NWC = 8, NWK = 1, CPW = 2; };
struct PanelSplit { static constexpr int NWC = 4, NWK = 2, CPW = 1; };
// Split shapes for one token block of 16-bit elements: with a single token block the registers leave room for
// three or four wavefronts per SIMD, and a launch of few workgroups (one per CU at most) streams faster with 12 or
// 16 wavefronts per workgroup than with 8 (4096 x 14336, 16 tokens: 1 / 2 / 4 / 8 masks 64.6 / 64.3 / 68.3 / 63.9 %
// of the HBM peak with two K-split wavefronts per column block, 72.8 / 71.2 / 69.5-70.8 / 65.1 % with 4 / 4 / 3 / 3;
// four with 4 masks measured 67.0 %).
struct PanelSplit3 { static constexpr int NWC = 4, NWK = 3, CPW = 1; };
struct PanelSplit4 { static constexpr int NWC = 4, NWK = 4, CPW = 1; };
// K-split wavefronts per column block of the split shape a launch of `tb` token blocks uses
__host__ __device__ constexpr int split_nwk(bool is_f32, int nmp, int tb)
{
    return (is_f32 || tb != 1 || nmp > 8) ? PanelSplit::NWK : nmp <= 2 ? PanelSplit4::NWK : PanelSplit3::NWK;
}
template <typename Tr, int NMP, int TB>
struct SplitShape {
    static constexpr int kNwk = split_nwk(Tr::ELEM_BYTES == 4, NMP, TB);
    typedef typename std::conditional<kNwk == 4, PanelSplit4,
                                      typename std::conditional<kNwk == 3, PanelSplit3, PanelSplit>::type>::type type;
};

struct StreamPlan {
    bool resident;
    bool wide;     // panel kernel: PanelWide (else PanelSplit)
    int tb;        // token blocks of 16 per workgroup
    int nw;        // resident kernel: wavefronts per workgroup, 1 << nw_shift
    int nw_shift;
    size_t lds;
    dim3 grid, block;
};

static StreamPlan plan_stream(const StreamParams &p, int elem_kind, int nmp, int sets)
{
    const bool is_f32 = elem_kind == kElemF32;
    constexpr size_t kLdsBudget = 56 * 1024;
    const int elem = is_f32 ? 4 : 2;
    const int tiles = is_f32 ? F32Traits::TILES : Bf16Traits::TILES;
    StreamPlan pl = {};
    // resident: one token block whose x rows (plus the reduction hand-over) fit the LDS budget
    const int tc = p.T < 16 ? p.T : 16;
    // wavefronts that split K: a power of two, at most MGLU_STREAM_MAX_WAVES, and few enough that each owns two chunks
    int nw_shift = 0;
    while ((2 << nw_shift) <= MGLU_STREAM_MAX_WAVES && (4 << nw_shift) <= p.NC) ++nw_shift;
    const int nw = 1 << nw_shift;
    // hand-over area: every wavefront's sums plus, for the shared epilogue, every wavefront's share
    const size_t red = nw > 1 ? (size_t)(nw * sets + nw) * 4 * tc * sizeof(f32x4) : 0;
    const size_t xb = (size_t)resident_x_frags_padded((p.NC * tiles * 4) << resident_row_shift(tc), nw_shift) * 16;
    if (p.T <= MGLU_RESIDENT_MAX_T && xb + red <= kLdsBudget) {
        pl.resident = true;
        pl.tb = 1;
        pl.nw = nw;
        pl.nw_shift = nw_shift;
        pl.lds = xb + red;
        pl.grid = dim3(p.NB, 1);
        pl.block = dim3(nw * kWave);
        return pl;
    }
    const int blocks = (int)ceil_div(p.T, 16);
    const int max_tb = stream_max_token_blocks(nmp, elem_kind);
    pl.resident = false;
    pl.tb = (blocks >= 4 && max_tb >= 4) ? 4 : (blocks >= 2 && max_tb >= 2) ? 2 : 1;
    pl.wide = ceil_div(p.NB, PanelWide::NWC) >= MGLU_PANEL_WIDE_MIN_WGS;
    const int nwc = pl.wide ? PanelWide::NWC : PanelSplit::NWC;
    const int nwk = pl.wide ? PanelWide::NWK : split_nwk(is_f32, nmp, pl.tb);
    const int cpw = pl.wide ? PanelWide::CPW : PanelSplit::CPW;
    const size_t xpanel = (size_t)2 * nwk * cpw * tiles * pl.tb * 1024;
    const size_t redp = (size_t)nwc * (nwk - 1) * sets * pl.tb * 1024;
    pl.lds = xpanel > redp ? xpanel : redp;
    pl.grid = dim3((unsigned)ceil_div(p.NB, nwc), (unsigned)ceil_div(p.T, 16 * pl.tb));
    pl.block = dim3(nwc * nwk * kWave);
    return pl;
}

// gfx950 has 160 KiB of LDS per CU; a kernel may use more than the default 64 KiB of dynamic LDS
// once it has been allowed to (asked once per kernel instantiation, not per launch).
constexpr int kMaxDynamicLds = 160 * 1024;

template <typename Tr, int NMP, int TB, int MODE, typename Shape>
static hipError_t launch_panel_one(const StreamParams &p, const StreamPlan &pl, hipStream_t stream)
{
    constexpr int NWC = Shape::NWC, NWK = Shape::NWK, CPW = Shape::CPW;
    if (p.describe) {   // name the instantiation instead of launching it
        snprintf(p.describe, p.describe_len, "stream_panel_kernel<%s, %d, %d, %d, %d, %d, %d>", traits_name<Tr>(), NMP,
                 TB, MODE, NWC, NWK, CPW);
        return hipSuccess;
    }
    auto kern = stream_panel_kernel<Tr, NMP, TB, MODE, NWC, NWK, CPW>;
    // one flag per instantiation (this function is a template over all of the kernel's parameters)
    static hipError_t allowed = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                    hipFuncAttributeMaxDynamicSharedMemorySize, kMaxDynamicLds);
    if (pl.lds > 64 * 1024 && allowed != hipSuccess) return allowed;
    hipLaunchKernelGGL(kern, pl.grid, pl.block, pl.lds, stream, p);
    return hipGetLastError();
}

template <typename Tr, int NMP, int MODE, int R, bool RX>
static hipError_t launch_resident(const StreamParams &p, const StreamPlan &pl, hipStream_t stream)
{
    if (p.describe) {
        snprintf(p.describe, p.describe_len, "stream_resident_kernel<%s, %d, %d, %d, %s>", traits_name<Tr>(), NMP, MODE, R,
                 RX ? "true" : "false");
        return hipSuccess;
    }
    hipLaunchKernelGGL((stream_resident_kernel<Tr, NMP, MODE, R, RX>), pl.grid, pl.block, pl.lds, stream, p.w, p.m, p.x,
                       p.NC, p.T, p.h, p.d, p.out, pl.nw_shift, p.n_masks, p.NB, p.w2, p.proj_t, p.proj_gate, p.proj_value,
                       p.gate_fn, p.mask_use, p.route);
    return hipGetLastError();
}

template <typename Tr, int NMP, int MODE, typename Shape>
static hipError_t launch_panel(const StreamParams &p, const StreamPlan &pl, hipStream_t stream)
{
    constexpr bool kIsBf16 = Tr::ELEM_BYTES == 2;
    constexpr bool kSplit = std::is_same<Shape, PanelSplit>::value;
    typedef typename std::conditional<kSplit, typename SplitShape<Tr, NMP, 1>::type, Shape>::type ShapeOne;
    if (pl.tb == 1) return launch_panel_one<Tr, NMP, 1, MODE, ShapeOne>(p, pl, stream);
    if constexpr (kIsBf16 && NMP <= 8) {
        if (pl.tb == 2) return launch_panel_one<Tr, NMP, 2, MODE, Shape>(p, pl, stream);
        if constexpr (NMP <= 2) {
            if (pl.tb == 4) return launch_panel_one<Tr, NMP, 4, MODE, Shape>(p, pl, stream);
        }
    }
    return hipErrorInvalidValue;
}

template <typename Tr, int NMP, int MODE>
static hipError_t launch_plan(const StreamParams &p, const StreamPlan &pl, hipStream_t stream)
{
    if (pl.resident) {
        if constexpr (MODE == kModeMglu && Tr::ELEM_BYTES == 2) {
            if ((long)p.NB * p.NC <= 256L * MGLU_RESIDENT_RX_MAX_CHUNKS_PER_CU)
                return launch_resident<Tr, NMP, MODE, MGLU_STREAM_RING, true>(p, pl, stream);
        }
        return launch_resident<Tr, NMP, MODE, MGLU_STREAM_RING, false>(p, pl, stream);
    }
    return pl.wide ? launch_panel<Tr, NMP, MODE, PanelWide>(p, pl, stream)
                   : launch_panel<Tr, NMP, MODE, PanelSplit>(p, pl, stream);
}

template <typename Tr, int MODE>
static hipError_t launch_nmp(const StreamParams &p, int nmp, const StreamPlan &pl, hipStream_t s)
{
    switch (nmp) {
    case 1: return launch_plan<Tr, 1, MODE>(p, pl, s);
    case 2: return launch_plan<Tr, 2, MODE>(p, pl, s);
    case 4: return launch_plan<Tr, 4, MODE>(p, pl, s);
    case 8: return launch_plan<Tr, 8, MODE>(p, pl, s);
    default: return launch_plan<Tr, 16, MODE>(p, pl, s);
    }
}

template <typename Tr>
static hipError_t launch_mode(const StreamParams &p, int mode, int nmp, const StreamPlan &pl, hipStream_t stream)
{
    switch (mode) {
    case kModeMglu: return launch_nmp<Tr, kModeMglu>(p, nmp, pl, stream);
    case kModeMgluVariant: return launch_nmp<Tr, kModeMgluVariant>(p, nmp, pl, stream);
    case kModeProjections: return launch_nmp<Tr, kModeProjections>(p, nmp, pl, stream);
    case kModeLinear: return launch_plan<Tr, 1, kModeLinear>(p, pl, stream);
    default: return launch_plan<Tr, 1, kModeSwiglu>(p, pl, stream);
    }
}

// Everything above is instantiated once per element type, each in a source file of its own
// (mglu_stream_bf16.hip, _f16.hip, _f32.hip) so that they compile side by side.
template <typename Tr>
static hipError_t launch_stream_t(const StreamParams &p, int elem, int mode, hipStream_t stream)
{
    const int nmp = (mode == kModeSwiglu || mode == kModeLinear) ? 1 : round_up_masks(p.n_masks);
    const StreamPlan pl = plan_stream(p, elem, nmp, sets_of(mode, nmp));
    return launch_mode<Tr>(p, mode, nmp, pl, stream);
}

}  // namespace mglu
