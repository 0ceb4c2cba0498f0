// Host-callable launchers of the MGLU kernels (internal to libmglu).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mglu_common.hpp"

namespace mglu {

struct StreamParams {
    const void *x;        // [T][h]
    const void *w;        // packed weights (SwiGLU: the gate matrix)
    const void *w2;       // SwiGLU only: packed value matrix
    const uint32_t *m;    // packed masks
    void *out;            // [T][d]
    float *proj_t;        // projections mode: [T][d], may be null
    float *proj_gate;     // [n_masks][T][d], may be null
    float *proj_value;    // [n_masks][T][d], may be null
    int T, h, d, n_masks;
    int NB;               // column blocks  = ceil(d / 16)
    int NC;               // reduction chunks = ceil(h / 128)
    int gate_fn;          // epilogue variant: see EpilogueParams
    int mask_use;
    const float *route;   // [T][n_masks] route weights, may be null
    char *describe;       // host only: if set, the launcher writes the kernel instantiation it would launch
    size_t describe_len;  //            here (as text) and launches nothing
};

struct PrefillParams {
    const void *x;        // [T][h] bf16
    const void *w;        // packed weights (SwiGLU: the gate matrix)
    const void *w2;       // SwiGLU only: packed value matrix
    const uint32_t *m;    // packed masks
    void *out;            // [T][d] bf16
    int T, h, d, n_masks;
    int NB, NC;
    int tiles_m, tiles_n; // filled in by the launcher
    int group_m;          // token tiles per L2 patch
    int gate_fn;          // epilogue variant: see EpilogueParams
    int mask_use;
    const float *route;   // [T][n_masks] route weights, may be null
    float *workspace;     // fp32 [T][d], needed with more than 8 masks (two launches of 8 masks each)
    // filled in by the launcher: which part of the layer's masks this launch covers
    int mask_chunk_bytes; // bytes from one chunk's mask words to the next chunk's
    int mask_offset;      // byte offset of this launch's masks inside a chunk's words
    int route_stride;     // mask count of the layer (row stride of `route`)
    const float *partial_in;   // fp32 [T][d] sum of the masks an earlier launch covered, added before rounding
    float *partial_out;        // if set, the fp32 sum goes here instead of `out`
    char *describe;       // host only: see StreamParams
    size_t describe_len;
};

// Routed layer on the planar mask format (mglu_routed.hip)
struct RoutedParams {
    const void *x;        // [T][h]
    const void *w;        // packed weights
    const uint32_t *m;    // planar packed masks
    void *out;            // [T][d]
    const float *route;   // [T][n_masks] route weights
    int T, h, d, n_masks;
    int NB, NC;
    int gate_fn;
    int k;                // non-zero weights per token the caller promises at most (sizes the kernel)
    char *describe;       // host only: see StreamParams
    size_t describe_len;
};

struct RouteParams {
    const void *x;        // [T][h]
    const void *wr;       // [h][n_masks], same element type as x
    float *weights;       // [T][n_masks]
    int T, h, n_masks, k;
};

struct PackParams {
    const void *src;      // W or mask bytes, layout per `nk`
    void *dst;
    int h, d, n_masks;
    int NB, NC;
    int nk;               // 0: [h][d] (masks [n][h][d]); 1: [d][h] (masks [n][d][h])
};

// Largest token-block count (blocks of 16 tokens) a workgroup of the streaming kernels handles per pass over W:
// what the 256-register budget of the panel kernel allows.  Beyond 16 x this many tokens the streaming kernels
// would read W once per group of token blocks, and the 16-bit types hand over to the MFMA-tiled kernel.
inline int stream_max_token_blocks(int nmp, int elem) { return elem == kElemF32 || nmp > 8 ? 1 : nmp <= 2 ? 4 : 2; }

// Whether the MFMA-tiled kernel runs a layer as two launches of 8 masks each (and needs the fp32 workspace):
// more than 8 masks and more tokens than the one 32-token tile that 17 accumulator sets leave registers for.
// (Up to 32 tokens one launch reads W once; two would read it twice for nothing.)
inline bool prefill_two_launches(int n_masks, int tokens) { return n_masks > 8 && tokens > 32; }

// `elem` is an Elem (mglu_common.hpp): the element type of x, W and out
hipError_t launch_stream(const StreamParams &p, int elem, int mode, hipStream_t stream);
hipError_t launch_stream_read(const void *buf, size_t bytes, uint32_t *sink, hipStream_t stream);

hipError_t launch_prefill(const PrefillParams &p, int elem, int mode, hipStream_t stream);   // 16-bit elements only

hipError_t launch_route_topk(const RouteParams &p, int elem, hipStream_t stream);

// false if the shape is outside what the routed kernel covers (more than 16 tokens, or rows of x beyond its LDS budget)
bool routed_supported(const RoutedParams &p, int elem);
hipError_t launch_routed(const RoutedParams &p, int elem, hipStream_t stream);

hipError_t launch_pack_weights(const PackParams &p, int elem, hipStream_t stream);
hipError_t launch_pack_masks(const PackParams &p, int elem, hipStream_t stream);
hipError_t launch_pack_masks_planar(const PackParams &p, int elem, hipStream_t stream);

}  // namespace mglu
