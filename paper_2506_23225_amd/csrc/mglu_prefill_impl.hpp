// MFMA-tiled MGLU kernel for prefill / large batches (bf16): compute-bound.
//
// The paper has no batched kernel; what it states for this regime is the cost model
// (Discussion, "Computational Cost": one dense contraction plus one per mask).  The layer
// is Eq. 3; the complement trick of Alg. 1 carries over: per output tile the kernel keeps
// 1 + n_m accumulator sets, t = x W and dsum_i = x (W with the sign of every gate element
// flipped), and the epilogue forms gate_i = (t - dsum_i)/2, value_i = (t + dsum_i)/2,
// sum_i swish(gate_i) * value_i in registers.  So the matrix cores do (1 + n_m) GEMMs'
// worth of work instead of the 2 n_m of the naive form, and W, the masks and x are each
// staged once per tile for all of them.
//
// Tiling (one workgroup = NW = 8 wavefronts = one CU at 2 wavefronts per SIMD, or NW = 4 and two per CU):
//   workgroup tile  BM = 16*TB tokens  x  BN = NW*16*CB columns
//   wavefront w owns CB column blocks of 16 columns, for all BM tokens
//   A operand (W): streamed straight from global memory in the packed tile order -- each
//     wavefront reads only its own column blocks, so LDS staging would buy no reuse
//   masks: read next to W, one chunk (128 k) of words at a time, applied in registers
//   B operand (x): shared by all wavefronts -> staged through LDS in B-fragment order by loads
//     that go from global memory straight to LDS (no registers, no LDS write instructions),
//     double-buffered per 128-k chunk, one barrier per chunk
//   MFMA: v_mfma_f32_16x16x32_bf16, 16 columns x 16 tokens per accumulator
// Workgroup ids are remapped so that the workgroups resident on one XCD (ids equal mod 8)
// cover a compact patch of tiles and share W / x through that XCD's L2.
#pragma once
#include <stdio.h>

#include <type_traits>

#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

#ifndef MGLU_PREFILL_AD1
#define MGLU_PREFILL_AD1 2   // tiles of W fetched ahead with one mask and in the two-matrix reference (two column blocks per wavefront)
#endif
#ifndef MGLU_PREFILL_AD_SMALL
#define MGLU_PREFILL_AD_SMALL 6   // tiles of W fetched ahead in the 4-wavefront shapes that have the registers for it
#endif

namespace mglu {

// In which tile of a chunk the s-th x piece of the next chunk is loaded / written to LDS.
#ifndef MGLU_PREFILL_XLOAD_TILE
#define MGLU_PREFILL_XLOAD_TILE(s, n) ((s) * 3 / (n))
#endif
// LDS buffers of one chunk of x each.  2: a chunk is staged while the one before it is multiplied, one
// barrier per chunk.  4: staged two chunks ahead, one barrier per two chunks, so that the wavefronts
// of a workgroup may drift a chunk apart instead of meeting after every chunk.
#ifndef MGLU_PREFILL_XBUF
#define MGLU_PREFILL_XBUF 2
#endif
constexpr int kPrefillXBuf = MGLU_PREFILL_XBUF;
#ifndef MGLU_PREFILL_MASK_MAJOR
#define MGLU_PREFILL_MASK_MAJOR 1
#endif
constexpr bool kPrefillMaskMajor = MGLU_PREFILL_MASK_MAJOR;
constexpr int kPrefillXAhead = kPrefillXBuf / 2;   // chunks between staging and use

// AD: how many tiles ahead of the multiply the A fragments are fetched.
// NW: wavefronts per workgroup.  8: one workgroup fills a CU (2 wavefronts per SIMD).  4: a CU holds two, and
// a launch of at most 256 such workgroups gives every wavefront a SIMD of its own -- for launches that would
// otherwise leave CUs idle while the busy ones run two wavefronts per SIMD.
template <typename Tr, int NMP, int CB, int TB, int MODE, int AD, int NW>
__global__ __launch_bounds__(NW *kWave) __attribute__((amdgpu_waves_per_eu(2, 2)))
void prefill_kernel(PrefillParams p)
{
    typedef typename Tr::frag frag;
    constexpr int SETS = sets_of(MODE, NMP);
    // ring entries: the tiles of one chunk, or of two chunks for a deep prefetch (a ring of four chunks with
    // the masks fetched as far ahead was measured too: no faster)
    constexpr int AR = AD <= 3 ? 4 : 8;
    constexpr int MR = 2;                       // mask ring entries (chunks): this chunk's and the next one's
    static_assert(AD < AR, "the fragment being multiplied must not be overwritten");
    constexpr long CHUNK_BYTES = (long)kColBlock * kChunkK * 2;
    // x fragments each wavefront stages per chunk (the last one only by the first wavefronts when the
    // TB * 4 fragments do not split evenly)
    constexpr int XPIECES = (TB * 4 + NW - 1) / NW;
    extern __shared__ f32x4 lds_raw[];
    frag *lds_x = reinterpret_cast<frag *>(lds_raw);   // [2][tile t<4][tb<TB][lane<64]
    // byte address of that array inside LDS, for the hand-placed reads
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)lds_raw;

    const int lane = threadIdx.x & 63;
    // the wavefront index is uniform over the wavefront: say so, and every address below splits into
    // a scalar base plus a 32-bit per-lane offset (no 64-bit vector arithmetic per load)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, q = lane >> 4;
    const uint32_t lane16 = lane * 16;

    // ---- XCD-aware tile order: ids equal mod 8 share an L2; give each XCD a band of column
    //      tiles and walk it in patches of p.group_m token tiles ----
    int tile_m, tile_n;
    {
        const int wg = blockIdx.x;
        const int xcd = wg & 7, local = wg >> 3;
        const int per_xcd = (p.tiles_n + 7) >> 3;         // column tiles per XCD band
        const int gm = p.group_m;
        const int patch = local / (gm * per_xcd);          // which group of token tiles
        const int in_patch = local - patch * gm * per_xcd;
        const int m0 = patch * gm;
        const int rows = min(gm, p.tiles_m - m0);          // last patch may be short
        tile_m = m0 + in_patch % rows;
        tile_n = xcd * per_xcd + in_patch / rows;
        if (tile_m >= p.tiles_m || tile_n >= p.tiles_n || in_patch / rows >= per_xcd) return;
    }
    const int tok0 = tile_m * (16 * TB);
    const int jb0 = (tile_n * NW + wave) * CB;   // first column block of this wavefront

    // column blocks past the end are clamped for the loads and dropped at the store
    const char *wbase[CB];       // scalar: start of the column block's weight stream
    const char *w2base[CB];
    const char *mbase[CB];       // scalar: start of its mask words
    // Only the 8-mask kernels are ever pointed at one half of a 16-mask layer (chunk stride and offset
    // from the launcher, fp32 hand-over in the epilogue); the others keep the constants.
    constexpr bool HALVES = NMP == 8 && (MODE == kModeMglu || MODE == kModeMgluVariant);
    const int mask_chunk_bytes = HALVES ? p.mask_chunk_bytes : kWave * NMP * 4;
    const int mask_offset = HALVES ? p.mask_offset : 0;
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const long jb = min(jb0 + cb, p.NB - 1);
        wbase[cb] = static_cast<const char *>(p.w) + jb * p.NC * CHUNK_BYTES;
        w2base[cb] = static_cast<const char *>(p.w2) + jb * p.NC * CHUNK_BYTES;
        mbase[cb] = reinterpret_cast<const char *>(p.m) + jb * p.NC * mask_chunk_bytes + mask_offset;
    }
    const uint32_t lane_m = mask_lane_bytes<NMP>(lane);

    f32x4 acc[SETS][CB][TB];
#pragma unroll
    for (int s = 0; s < SETS; ++s)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) acc[s][cb][tb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // ---- x staging: wavefront w copies fragments idx = w + NW s (idx = tb * 4 + t) of a chunk:
    //      lane (r, q) moves x[tok0 + 16 tb + r][128 kc + 32 t + 8 q .. + 8) to LDS slot
    //      (t * TB + tb) * 64 + lane, the order the B operand is read in.  Token rows past T are
    //      clamped to the last row (their outputs are never stored) and k past d_model to the
    //      row's last fragment (W is zero-padded there, so whatever finite x is read adds 0). ----
    const char *xbase = static_cast<const char *>(p.x) + (long)tok0 * p.h * 2;   // scalar
    const uint32_t klim = (uint32_t)(p.h - 8) * 2;
    uint32_t xrow[XPIECES];      // per piece: byte offset of this lane's token row from xbase
#pragma unroll
    for (int s = 0; s < XPIECES; ++s) {
        const int tb = (wave + NW * s) >> 2;
        xrow[s] = (uint32_t)(min(tok0 + 16 * tb + r, p.T - 1) - tok0) * (uint32_t)(p.h * 2);
    }
    // One fragment of x goes from global memory straight to LDS (no registers in between): the load
    // takes a per-lane byte offset into a buffer and a wavefront-uniform LDS address, and lane l's 16
    // bytes land at that address + 16 l -- exactly a B fragment's slot order.  The buffer is this
    // workgroup's token rows (offsets past its end would read as zero; the clamps keep them inside).
    const __amdgpu_buffer_rsrc_t xrsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<char *>(xbase), 0, (min(tok0 + 16 * TB, p.T) - tok0) * p.h * 2, 0x00020000);
    auto stage_x = [&](int kc, int buf, int s) __attribute__((always_inline)) {
        const int idx = wave + NW * s;
        const int tb = idx >> 2, t = idx & 3;
        const uint32_t kb = min((uint32_t)(kc * kChunkK + 32 * t) * 2 + q * 16, klim);
        frag *dst = lds_x + ((buf * 4 + t) * TB + tb) * kWave;   // uniform over the wavefront
        if (TB * 4 % NW == 0 || idx < TB * 4)   // uniform; skipping the last piece only makes the wait below stricter
            __builtin_amdgcn_raw_ptr_buffer_load_lds(xrsrc, (__attribute__((address_space(3))) void *)dst, 16,
                                                 (int)(xrow[s] + kb), 0, 0, 0);
    };

    // ---- A ring: entry t holds the fragments of tile t of the current (or next) chunk ----
    frag aw[AR][CB];
    frag aw2[MODE == kModeSwiglu ? AR : 1][CB];
    uint32_t mk[MR][CB][NMP];  // mask words of the current chunk and the MR - 1 after it

    auto load_a = [&](int kc, int t, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            aw[slot][cb] = *reinterpret_cast<const frag *>(wbase[cb] + (long)kc * CHUNK_BYTES + t * 1024 + lane16);
            if constexpr (MODE == kModeSwiglu)
                aw2[slot][cb] =
                    *reinterpret_cast<const frag *>(w2base[cb] + (long)kc * CHUNK_BYTES + t * 1024 + lane16);
        }
    };
    // 16 masks: the words of a chunk are fetched in two parts -- part 0 = pieces 0 and 2 (tiles 0, 1 of either
    // 8-mask half), part 1 = pieces 1 and 3 (tiles 2, 3) -- so that fewer than 32 mask registers are live at a time
    // (32 spilled more).  Where W is fetched 2 tiles ahead (workgroups share it through L2) so is each part: 16
    // live.  The shapes that stream W from HBM with a deeper prefetch keep the masks a whole chunk ahead, part
    // by part: 24 live.
    constexpr bool SPLIT16 = NMP == 16 && MODE != kModeSwiglu && MODE != kModeLinear;
    constexpr bool SPLIT16_NEAR = SPLIT16 && AD <= 2;
    auto load_masks = [&](int kc, int slot, int part = -1) __attribute__((always_inline)) {
        if constexpr (MODE != kModeSwiglu && MODE != kModeLinear) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                const uint32_t *mp =
                    reinterpret_cast<const uint32_t *>(mbase[cb] + (long)kc * mask_chunk_bytes + lane_m);
                if constexpr (NMP >= 8) {
#pragma unroll
                    for (int piece = 0; piece < NMP / 4; ++piece) {
                        if (part >= 0 && (piece & 1) != part) continue;   // compile time after inlining
                        u32x4 a = *reinterpret_cast<const u32x4 *>(reinterpret_cast<const char *>(mp) + piece * kMaskPieceBytes);
#pragma unroll
                        for (int i = 0; i < 4; ++i) mk[slot][cb][4 * piece + i] = a[i];
                    }
                } else if constexpr (NMP == 4) {
                    u32x4 a = *reinterpret_cast<const u32x4 *>(mp);
#pragma unroll
                    for (int i = 0; i < 4; ++i) mk[slot][cb][i] = a[i];
                } else if constexpr (NMP == 2) {
                    u32x2 a = *reinterpret_cast<const u32x2 *>(mp);
                    mk[slot][cb][0] = a.x; mk[slot][cb][1] = a.y;
                } else {
                    mk[slot][cb][0] = *mp;
                }
            }
        }
    };

    constexpr int A_LOADS = CB * (MODE == kModeSwiglu ? 2 : 1);   // load instructions of one load_a / load_masks
    constexpr int M_LOADS = (MODE == kModeSwiglu || MODE == kModeLinear) ? 0 : CB * (NMP >= 8 ? NMP / 4 : 1);
    constexpr int M_PROLOGUE = SPLIT16_NEAR ? M_LOADS / 2 : (MR - 1) * M_LOADS;   // mask loads issued before the loop
    auto wait_vm = [](auto n) __attribute__((always_inline)) {
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(decltype(n)::value) : "memory");
    };

    // ---- prologue: stage the first chunk(s) of x, start the A ring and the masks ----
    const int last = p.NC - 1;
    {
#pragma unroll
        for (int c = 0; c < kPrefillXAhead; ++c)
#pragma unroll
            for (int s = 0; s < XPIECES; ++s) stage_x(min(c, last), c, s);
        __builtin_amdgcn_sched_barrier(0);   // the x loads stay the oldest ones in flight
#pragma unroll
        for (int c = 0; c < MR - 1; ++c) load_masks(min(c, last), c, SPLIT16_NEAR ? 0 : -1);
#pragma unroll
        for (int t = 0; t < AD; ++t) load_a(min(t / 4, last), t % 4, t % AR);
    }
    // Loads complete in issue order, so "at most the loads issued after them outstanding" means the x
    // fragments are in LDS; the compiler does not know that the hand-placed LDS reads depend on them.
    wait_vm(std::integral_constant<int, M_PROLOGUE + AD * A_LOADS>{});
    __builtin_amdgcn_s_barrier();

    // One chunk of the K loop; PHASE = kc modulo the unroll (compile time): it fixes which entry of mk[]
    // holds this chunk's masks and where its tiles sit in the ring.
    auto chunk_step = [&](int kc, auto phase_tag) __attribute__((always_inline)) {
        constexpr int PHASE = decltype(phase_tag)::value;
        constexpr int MS = PHASE % MR;
        constexpr int RS = (4 * PHASE) % AR;       // ring slot of this chunk's first tile
        const int buf = kc & (kPrefillXBuf - 1);
        const int kn = min(kc + MR - 1, last);   // the chunk whose masks are fetched now, clamped: always in bounds
        const int kx = min(kc + kPrefillXAhead, last);   // the chunk of x staged during this one
        // B fragments are read from LDS one pair of token blocks ahead of the MFMAs that use them
        // (the compiler, left alone, issues each read right before its use and eats the LDS latency
        // three times per tile).  The first pair of a chunk cannot be fetched before the barrier.
        constexpr int PAIRS = TB / 2;
        // The reads are written as assembly so that they stay where they are put; the matching
        // waits name the registers they release, which orders every use after them.  (lgkmcnt
        // counts LDS operations in order, so "at most 2 newer ones outstanding" means the pair
        // before them has landed; anything else in flight only makes the wait stricter.)
        const uint32_t xchunk = lds_base + (uint32_t)(buf * 4 * TB * kWave + lane) * 16u;
        auto read_pair = [&](frag (&b)[2], int t, int pi) __attribute__((always_inline)) {
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(b[0]) : "v"(xchunk), "n"((t * TB + 2 * pi) * 1024));
            asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(b[1]) : "v"(xchunk), "n"((t * TB + 2 * pi + 1) * 1024));
        };
        // Mask-major tiles (four masks): all B fragments of a tile stay in registers, one set per tile
        // parity, and the sets are multiplied one after the other -- so mask i + 1's operand is prepared
        // in the issue slots between the MFMAs of mask i instead of ahead of the whole tile.  Worth
        // about 1 % there; with eight masks the second set of B fragments no longer fits the registers.
        constexpr bool MASK_MAJOR =
            kPrefillMaskMajor && (TB == 6 || TB == 3) && MODE != kModeSwiglu && MODE != kModeLinear;
        static_assert(TB % 2 == 0 || MASK_MAJOR, "token blocks are processed in pairs");
        auto read_tile = [&](frag (&b)[TB], int t) __attribute__((always_inline)) {
#pragma unroll
            for (int tb = 0; tb < TB; ++tb)
                asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(b[tb]) : "v"(xchunk), "n"((t * TB + tb) * 1024));
        };
        // wait until at most `newer` LDS operations issued after fragment b are outstanding, then release b
        auto wait_frag = [&](frag &b, int newer) __attribute__((always_inline)) {
            asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(b) : "n"(newer));
        };
        frag btile[MASK_MAJOR ? 2 : 1][TB];
        // Two pairs of B fragments used in turn: step n of a chunk multiplies bp[n & 1] while bp[(n + 1) & 1]
        // is being read.  The parity is a compile-time constant of the unrolled code, so every read is
        // waited for in the very registers it writes (no register copy of a read still in flight); a
        // chunk has an even number of steps, so every chunk starts with bp[0].
        frag bp[2][2];
        if constexpr (MASK_MAJOR) read_tile(btile[0], 0);
        else read_pair(bp[0], 0, 0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            // Issue this tile's prefetches first: pieces of the next chunk's x (stored one tile
            // later), the A fragments AD tiles ahead, and once per chunk the next chunk's masks.
            // The scheduling fence keeps the compiler from sinking these loads down to their
            // first use, which would expose the whole memory latency.
#pragma unroll
            for (int s = 0; s < XPIECES; ++s)
                if (MGLU_PREFILL_XLOAD_TILE(s, XPIECES) == t)
                    stage_x(kx, (kc + kPrefillXAhead) & (kPrefillXBuf - 1), s);
            __builtin_amdgcn_sched_barrier(0);   // x first: the wait at the end of the chunk counts on it
            load_a(min(kc + (t + AD) / 4, last), (t + AD) % 4, (RS + t + AD) % AR);
            if constexpr (SPLIT16_NEAR) {
                if (t == 0) load_masks(kc, MS, 1);
                if (t == 2) load_masks(kn, (MS + MR - 1) % MR, 0);
            } else if constexpr (SPLIT16) {
                if (t == 0) load_masks(kn, (MS + MR - 1) % MR, 0);
                if (t == 2) load_masks(kn, (MS + MR - 1) % MR, 1);
            } else {
                if (t == 0) load_masks(kn, (MS + MR - 1) % MR);
            }
            __builtin_amdgcn_sched_barrier(0);

            if constexpr (MASK_MAJOR) {
                frag (&b)[TB] = btile[t & 1];
                frag var[2][CB];
                constexpr int PER_SET = TB * CB;             // MFMAs of one set
                constexpr int FLIP_VALU = 6 * CB;            // vector instructions of one mask's operand
                constexpr int PER_GAP = (FLIP_VALU + PER_SET - 1) / PER_SET;
                // issue order of one set: its MFMAs one by one, the next operand's instructions in the gaps
                auto interleave = [&](bool with_flip) __attribute__((always_inline)) {
                    int left = with_flip ? FLIP_VALU : 0;
#pragma unroll
                    for (int k = 0; k < PER_SET; ++k) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                        if (left >= 2 && PER_GAP >= 2) __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);
                        else if (left >= 1) __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);
                        left -= left >= PER_GAP ? PER_GAP : left;
                    }
                };
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) var[0][cb] = Tr::template flip<NMP>(aw[(RS + t) % AR][cb], mk[MS][cb], t, 0);
                if (t == 0) {
                    // this tile's reads were issued right after the barrier: take the fragments as they land
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) {
                        wait_frag(b[tb], TB - 1 - tb);
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) acc[0][cb][tb] = Tr::mma(aw[(RS + t) % AR][cb], b[tb], acc[0][cb][tb]);
                    }
                    read_tile(btile[1], 1);
                } else {
                    // read the next tile's fragments now; this tile's were issued a tile ago
                    if (t + 1 < 4) read_tile(btile[(t + 1) & 1], t + 1);
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb) wait_frag(b[tb], t + 1 < 4 ? TB : 0);
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb) acc[0][cb][tb] = Tr::mma(aw[(RS + t) % AR][cb], b[tb], acc[0][cb][tb]);
                }
                interleave(true);
#pragma unroll
                for (int i = 0; i < NMP; ++i) {
                    if (i + 1 < NMP) {
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb)
                            var[(i + 1) & 1][cb] = Tr::template flip<NMP>(aw[(RS + t) % AR][cb], mk[MS][cb], t, i + 1);
                    }
#pragma unroll
                    for (int tb = 0; tb < TB; ++tb)
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb)
                            acc[1 + i][cb][tb] = Tr::mma(var[i & 1][cb], b[tb], acc[1 + i][cb][tb]);
                    interleave(i + 1 < NMP);
                }
            } else if constexpr (TB == 2 && MODE != kModeSwiglu && MODE != kModeLinear) {
                // Many masks, one pair of token blocks: each mask's operand is prepared right before its
                // two MFMAs and dropped after them (all variants at once would not fit the registers);
                // the issue-order groups keep the compiler from gathering the preparation up front.
                const bool more = t + 1 < 4;
                frag (&bcur)[2] = bp[t & 1];
                if (more) {
                    read_pair(bp[(t + 1) & 1], t + 1, 0);
                    asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(bcur[0]), "+v"(bcur[1]));
                } else {
                    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bcur[0]), "+v"(bcur[1]));
                }
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
#pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2) acc[0][cb][h2] = Tr::mma(aw[(RS + t) % AR][cb], bcur[h2], acc[0][cb][h2]);
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
#pragma unroll
                    for (int i = 0; i < NMP; ++i) {
                        const frag wf = Tr::template flip<NMP>(aw[(RS + t) % AR][cb], mk[MS][cb], t, i);
#pragma unroll
                        for (int h2 = 0; h2 < 2; ++h2) acc[1 + i][cb][h2] = Tr::mma(wf, bcur[h2], acc[1 + i][cb][h2]);
                        __builtin_amdgcn_sched_group_barrier(0x002, 8, 0);
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    }
                }
            } else {
                // operand variants of this tile: W itself and W with mask i's gate elements negated
                frag var[SETS][CB];
    #pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    var[0][cb] = aw[(RS + t) % AR][cb];
                    if constexpr (MODE == kModeSwiglu) {
                        var[1][cb] = aw2[(RS + t) % AR][cb];
                    } else if constexpr (MODE != kModeLinear) {
    #pragma unroll
                        for (int i = 0; i < NMP; ++i) var[1 + i][cb] = Tr::template flip<NMP>(aw[(RS + t) % AR][cb], mk[MS][cb], t, i);
                    }
                }
    #pragma unroll
                for (int pi = 0; pi < PAIRS; ++pi) {
                    const bool more = (pi + 1 < PAIRS) || (t + 1 < 4);
                    static_assert(MASK_MAJOR || (4 * PAIRS) % 2 == 0, "a chunk must have an even number of steps");
                    frag (&bcur)[2] = bp[(t * PAIRS + pi) & 1];
                    if (more) {
                        read_pair(bp[(t * PAIRS + pi + 1) & 1], pi + 1 < PAIRS ? t : t + 1, pi + 1 < PAIRS ? pi + 1 : 0);
                        asm volatile("s_waitcnt lgkmcnt(2)" : "+v"(bcur[0]), "+v"(bcur[1]));
                    } else {
                        asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(bcur[0]), "+v"(bcur[1]));
                    }
    #pragma unroll
                    for (int h2 = 0; h2 < 2; ++h2)
    #pragma unroll
                        for (int s = 0; s < SETS; ++s)
    #pragma unroll
                            for (int cb = 0; cb < CB; ++cb)
                                acc[s][cb][2 * pi + h2] = Tr::mma(var[s][cb], bcur[h2], acc[s][cb][2 * pi + h2]);
                }
            }
        }
        // the chunk's x fragments have landed in LDS once only the loads issued after the last of them
        // may still be outstanding (the A fragments of the tiles from that one on, and the masks if
        // that was the chunk's first tile)
        constexpr int XL = MGLU_PREFILL_XLOAD_TILE(XPIECES - 1, XPIECES);
        constexpr int M_AFTER_X = SPLIT16 ? ((XL == 0 ? 1 : 0) + (XL <= 2 ? 1 : 0)) * (M_LOADS / 2) : (XL == 0 ? M_LOADS : 0);
        wait_vm(std::integral_constant<int, (4 - XL) * A_LOADS + M_AFTER_X>{});
        // with two buffers every chunk ends in a barrier; with four only every second one (a buffer
        // is written two chunks after its last read and read two chunks after it was written, and
        // one barrier lies in between either way)
        if (kPrefillXBuf == 2 || (PHASE & 1) == 1) __builtin_amdgcn_s_barrier();
    };

    // the loop body covers two chunks, so that every chunk's place in the rings is known at compile time
    int kc = 0;
    for (; kc + 2 <= p.NC; kc += 2) {
        chunk_step(kc, std::integral_constant<int, 0>{});
        chunk_step(kc + 1, std::integral_constant<int, 1>{});
    }
    if (kc < p.NC) chunk_step(kc, std::integral_constant<int, 0>{});

    // ---- epilogue (Eq. 3): lane (r, q) holds token 16 tb + r, columns 4 q .. 4 q + 3 of each block ----
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int jb = jb0 + cb;
        if (jb >= p.NB) continue;
        const int j0 = jb * kColBlock + 4 * q;
        if (j0 >= p.d) continue;
        const bool full = (j0 + 3 < p.d) && ((p.d & 3) == 0);
#pragma unroll
        for (int tb = 0; tb < TB; ++tb) {
            const long tok = (long)tok0 + 16 * tb + r;
            if (tok >= p.T) continue;
            // plain mode: all NMP masks, a compile-time bound (a padding mask is all-value: its sum
            // equals t bit for bit, its gate is 0 and its term exactly 0)
            const EpilogueParams ep = MODE == kModeMgluVariant
                                          ? EpilogueParams{p.n_masks, p.gate_fn, p.mask_use, p.route, p.route_stride}
                                          : EpilogueParams{NMP, 0, 0, nullptr, 0};
            float rw[NMP];
            route_weights<NMP>(ep, tok, true, rw);
            f32x4 y;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if constexpr (MODE == kModeSwiglu) {
                    y[c] = swish(acc[0][cb][tb][c]) * acc[1][cb][tb][c];
                } else if constexpr (MODE == kModeLinear) {
                    y[c] = acc[0][cb][tb][c];
                } else {
                    float ds[NMP];
#pragma unroll
                    for (int i = 0; i < NMP; ++i) ds[i] = acc[1 + i][cb][tb][c];
                    y[c] = mglu_mix<NMP, MODE == kModeMglu>(ep, rw, acc[0][cb][tb][c], ds);
                }
            }
            const long o = tok * p.d + j0;
            // a layer of more than 8 masks runs as two launches: the first leaves its fp32 sum in the
            // workspace, the second adds it before the one rounding to the output type
            if constexpr (HALVES) {
                if (p.partial_in) {   // uniform
                    if (full) {
                        y += *reinterpret_cast<const f32x4 *>(p.partial_in + o);
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (j0 + c < p.d) y[c] += p.partial_in[o + c];
                    }
                }
                if (p.partial_out) {  // uniform
                    if (full) {
                        *reinterpret_cast<f32x4 *>(p.partial_out + o) = y;
                    } else {
#pragma unroll
                        for (int c = 0; c < 4; ++c)
                            if (j0 + c < p.d) p.partial_out[o + c] = y[c];
                    }
                    continue;
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

template <typename Tr, int NMP, int CB, int TB, int MODE, int AD, int NW>
static hipError_t launch_prefill_one(PrefillParams p, hipStream_t stream)
{
    const int bm = 16 * TB, bn = NW * kColBlock * CB;
    p.tiles_m = (int)ceil_div(p.T, bm);
    p.tiles_n = (int)ceil_div(p.d, bn);
    p.group_m = p.tiles_m < 8 ? p.tiles_m : 8;
    // every XCD gets per_xcd column tiles x tiles_m token tiles; ids beyond a band's end return at once
    const int per_xcd = (p.tiles_n + 7) / 8;
    const long wgs = (long)8 * per_xcd * p.tiles_m;
    const size_t lds = (size_t)kPrefillXBuf * 4 * TB * kWave * sizeof(f32x4);
    if (p.mask_chunk_bytes == 0) {   // the launch covers all the layer's masks
        p.mask_chunk_bytes = kWave * NMP * 4;
        p.route_stride = p.n_masks;
    }
    if (p.describe) {   // name the instantiation instead of launching it
        snprintf(p.describe, p.describe_len, "prefill_kernel<%s, %d, %d, %d, %d, %d, %d>%s",
                 traits_name<Tr>(), NMP, CB, TB, MODE, AD, NW, p.partial_in ? " twice" : "");
        return hipSuccess;
    }
    auto kern = prefill_kernel<Tr, NMP, CB, TB, MODE, AD, NW>;
    if (lds > 64 * 1024) {   // beyond the default dynamic LDS limit: allowed once per kernel
        static hipError_t allowed = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                        hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (allowed != hipSuccess) return allowed;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)wgs), dim3(NW * kWave), lds, stream, p);
    return hipGetLastError();
}

// ---- tile shape per launch ---------------------------------------------------------------------
// A wavefront's tile is 16 CB columns x 16 TB tokens, a workgroup's NW times as wide.  Taller and wider
// tiles load W and x less often per multiply, and that is what the loop's speed (and the clock the chip
// holds) responds to; smaller tiles and 4-wavefront workgroups fill the chip when the launch is small.
// Each kernel family lists its shapes, largest first; the launcher takes the one with the least
// estimated time: per-wavefront work x the wavefronts that share the busiest SIMD, one after the other.
// AD: tiles of W fetched ahead.  2 where workgroups of several token tiles share W through L2; 6 (an
// 8-entry ring) in the 4-wavefront shapes, whose launches have one or two token tiles and stream W
// straight from HBM with a single wavefront per SIMD to cover its latency.
template <int CB_, int TB_, int NW_, int AD_>
struct Tile { static constexpr int CB = CB_, TB = TB_, NW = NW_, AD = AD_; };

template <typename S>
static double prefill_cost(const PrefillParams &p)
{
    constexpr long kChipCUs = 256;
    const long wgs = ceil_div(p.T, 16 * S::TB) * ceil_div(p.d, S::NW * kColBlock * S::CB);
    const double work = S::TB * S::CB;   // MFMAs of a wavefront per k step and accumulator set
    double t;
    if (S::NW == 8) {
        t = (double)ceil_div(wgs, kChipCUs) * 2.0 * work;   // one workgroup per CU, two wavefronts per SIMD
    } else {
        // two workgroups per CU; up to 256 of them get a CU each (a wavefront alone on its SIMD runs a
        // little below twice the speed of two that share one)
        const long full = wgs / (2 * kChipCUs), rest = wgs % (2 * kChipCUs);
        t = full * 2.0 * work + (rest == 0 ? 0.0 : rest <= kChipCUs ? 1.2 * work : 2.0 * work);
        t *= 1.03;                                           // x is staged twice as often per multiply
    }
    // fewer multiplies per loaded fragment: measured 3-8 % from 96 to 128 tokens at four masks
    return t * (work >= 8 ? 1.0 : work >= 6 ? 1.05 : 1.12);
}

template <typename Tr, int NMP, int MODE, typename... Shapes>
static hipError_t launch_prefill_best(const PrefillParams &p, hipStream_t stream)
{
    int best = 0, i = 0;
    double best_cost = 0.0;
    auto consider = [&](double c) {
        if (i == 0 || c < best_cost) { best = i; best_cost = c; }   // ties go to the earlier (larger) shape
        ++i;
    };
    (consider(prefill_cost<Shapes>(p)), ...);
    hipError_t result = hipErrorInvalidValue;
    i = 0;
    auto launch_if = [&](auto shape) {
        typedef decltype(shape) S;
        if (i++ == best) result = launch_prefill_one<Tr, NMP, S::CB, S::TB, MODE, S::AD, S::NW>(p, stream);
    };
    (launch_if(Shapes{}), ...);
    return result;
}

template <typename Tr, int MODE>
static hipError_t launch_prefill_masks(const PrefillParams &p, hipStream_t stream)
{
    // accumulators (1 + n_m sets of CB x TB x 4 registers) must fit 256 registers with the operands
    switch (round_up_masks(p.n_masks)) {
    case 1: return launch_prefill_best<Tr, 1, MODE, Tile<2, 8, 8, MGLU_PREFILL_AD1>, Tile<2, 8, 4, MGLU_PREFILL_AD_SMALL>>(p, stream);
    case 2: return launch_prefill_best<Tr, 2, MODE, Tile<1, 8, 8, 2>, Tile<1, 8, 4, MGLU_PREFILL_AD_SMALL>>(p, stream);
    case 4: return launch_prefill_best<Tr, 4, MODE, Tile<1, 8, 8, 2>, Tile<1, 6, 8, 2>, Tile<1, 8, 4, 3>, Tile<1, 4, 4, MGLU_PREFILL_AD_SMALL>>(p, stream);
    case 8: return launch_prefill_best<Tr, 8, MODE, Tile<1, 4, 8, 2>, Tile<1, 4, 4, 3>>(p, stream);
    default: {
        // 9 to 16 masks, more than 32 tokens: two launches of the 8-mask kernels, one per half of the 16-mask format (two 8-mask
        // blocks side by side in every chunk).  The first leaves the fp32 sum of its masks' terms in the
        // workspace, the second adds its own and rounds once.  18 accumulator sets' worth of multiplies
        // instead of 17, at 64-token wavefront tiles instead of the 32 tokens that 17 sets would leave
        // registers for (measured: 44 % of the matrix peak in one launch, 61 % for an 8-mask launch).
        if (!prefill_two_launches(p.n_masks, p.T))
            return launch_prefill_best<Tr, 16, MODE, Tile<1, 2, 8, 2>, Tile<1, 2, 4, 3>>(p, stream);
        if (!p.workspace) return hipErrorInvalidValue;
        PrefillParams a = p, b = p;
        a.mask_chunk_bytes = b.mask_chunk_bytes = kWave * 16 * 4;
        a.route_stride = b.route_stride = p.n_masks;
        a.n_masks = 8;
        a.mask_offset = 0;
        a.partial_out = p.workspace;
        b.n_masks = p.n_masks - 8;
        b.mask_offset = kWave * 8 * 4;
        b.partial_in = p.workspace;
        if (p.route) b.route = p.route + 8;
        if (!p.describe) {
            const hipError_t e = launch_prefill_best<Tr, 8, MODE, Tile<1, 4, 8, 2>, Tile<1, 4, 4, 3>>(a, stream);
            if (e != hipSuccess) return e;
        }
        return launch_prefill_best<Tr, 8, MODE, Tile<1, 4, 8, 2>, Tile<1, 4, 4, 3>>(b, stream);
    }
    }
}

template <typename Tr>
static hipError_t launch_prefill_t(const PrefillParams &p, int mode, hipStream_t stream)
{
    if (mode == kModeSwiglu) return launch_prefill_one<Tr, 1, 2, 8, kModeSwiglu, MGLU_PREFILL_AD1, 8>(p, stream);
    // plain projection (one accumulator set): 4 column blocks per wavefront on full launches -- twice the MFMAs
    // per loaded fragment, 51-53 % of peak instead of 40-43 % on the 14336 -> 4096 projection
    if (mode == kModeLinear)
        return launch_prefill_best<Tr, 1, kModeLinear, Tile<4, 8, 8, 2>, Tile<2, 8, 8, 2>, Tile<2, 8, 4, MGLU_PREFILL_AD_SMALL>>(p, stream);
    if (mode == kModeMgluVariant) return launch_prefill_masks<Tr, kModeMgluVariant>(p, stream);
    return launch_prefill_masks<Tr, kModeMglu>(p, stream);
}

}  // namespace mglu
