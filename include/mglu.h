/*
 * libmglu -- forward pass of the Masked Gated Linear Unit (MGLU) on AMD MI355X (gfx950).
 *
 *   out[tau][j] = sum_{i=0}^{n_masks-1} swish( gate_i[tau][j] ) * value_i[tau][j]
 *   gate_i [tau][j] = sum_k x[tau][k] * W[k][j] * M_i[k][j]
 *   value_i[tau][j] = sum_k x[tau][k] * W[k][j] * (1 - M_i[k][j])
 *   swish(z) = z * sigmoid(z)
 *
 * This is Eq. 3 of the paper (the Mixture-of-Element-wise-Gating form; Eq. 2 is
 * the n_masks = 1 case), with k in [0, d_model) the hidden index h, j in
 * [0, d_ff) the intermediate index d, a mask bit of 1 sending the weight element
 * to the gate branch (Eq. 2; Alg. 1).  No bias, plain sum over the masks.
 *
 * As in the paper's FlashMGLU (section "FlashMGLU: Efficient Kernel
 * Implementation of MGLUs", Alg. 1) W is read once per call, the masks are
 * bit-packed (one bit per mask per weight element, the figure the paper's
 * memory-load table counts), the unmasked sum and one further sum per mask are
 * accumulated together, each value branch comes from the complement, and the
 * Swish, the products and the sum over masks happen on chip before the single
 * store of `out`.
 *
 * Conventions for every call
 *   - Every pointer named "dev" is DEVICE memory owned by the caller; the
 *     library allocates nothing, never copies to the host and never
 *     synchronises.  All work is enqueued on `stream` (a hipStream_t passed as
 *     void*; NULL is the default stream).
 *   - Device pointers must be 16-byte aligned.
 *   - Errors come back as mglu_status; mglu_last_error() gives the text of the
 *     calling thread's last failure.  A call that fails enqueues nothing.
 *   - The packed formats are opaque, produced only by the pack calls below and
 *     consumed only by this library version (mglu_format_version()).
 *   - Weights and masks are fixed at inference (paper, end of the "MoEG
 *     Variant" paragraph), so packing is a one-time set-up step, not part of
 *     the per-token path.
 */
#ifndef MGLU_H
#define MGLU_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MGLU_OK = 0,
    MGLU_ERR_INVALID_ARG = 1,  /* null pointer, misaligned pointer, non-positive size, bad enum */
    MGLU_ERR_UNSUPPORTED = 2,  /* valid in principle, not built (e.g. n_masks > 16) */
    MGLU_ERR_WORKSPACE = 3,    /* workspace missing or smaller than the query says */
    MGLU_ERR_HIP = 4           /* the HIP runtime refused a launch */
} mglu_status;

/* Element type of x, W and out.  Accumulation is always fp32. */
typedef enum {
    MGLU_F32 = 0,
    MGLU_BF16 = 1,
    MGLU_F16 = 2   /* IEEE binary16, the precision of the paper's own kernels */
} mglu_dtype;

/* How the caller's UNPACKED weight matrix and mask planes are laid out (row-major):
 *   MGLU_W_KN: W [d_model][d_ff],  masks [n_masks][d_model][d_ff]   (the paper's math, W in R^{h x d})
 *   MGLU_W_NK: W [d_ff][d_model],  masks [n_masks][d_ff][d_model]   (the paper's kernel, A [M x N] with K contiguous)
 * Only the pack calls and mglu_forward_bool read it. */
typedef enum { MGLU_W_KN = 0, MGLU_W_NK = 1 } mglu_layout;

typedef struct {
    int32_t tokens;      /* T >= 1: rows of x and out (ignored by the pack calls) */
    int32_t d_model;     /* h >= 1: reduction length */
    int32_t d_ff;        /* d >= 1: output width */
    int32_t n_masks;     /* n_m in [1, 16] */
    mglu_dtype dtype;
    mglu_layout w_layout;
} mglu_desc;

/* Bump whenever a packed format changes. */
int mglu_format_version(void);

/* ---- one-time set-up: packing (paper: "Packs mask bits", FlashMGLU section) ------------- */

/* Bytes of the packed weight buffer for (d_model, d_ff, dtype); 0 on a bad descriptor.
 * Equals the unpacked size whenever d_ff is a multiple of 16 and d_model of 128;
 * otherwise the matrix is zero-padded up to those multiples. */
size_t mglu_packed_weight_bytes(const mglu_desc *desc);

/* Re-tiles W into the order the kernels stream it in (each wavefront load is one
 * contiguous 1 KiB run).  W_dev: [d_model][d_ff] or [d_ff][d_model] per desc->w_layout,
 * element type desc->dtype.  packed_dev: mglu_packed_weight_bytes(desc) bytes, fully
 * overwritten. */
mglu_status mglu_pack_weights(const mglu_desc *desc, const void *W_dev, void *packed_dev, void *stream);

/* Bytes of the packed mask buffer: one bit per mask per (padded) weight element, with
 * n_masks rounded up to 1, 2, 4, 8 or 16 (the padding planes are all-zero, i.e. all-value,
 * and contribute exactly 0 to Eq. 3).  0 on a bad descriptor. */
size_t mglu_packed_mask_bytes(const mglu_desc *desc);

/* Packs n_masks planes of bytes (0 = value branch, non-zero = gate branch) into bit
 * planes in register-native order.  masks_dev: [n_masks][d_model][d_ff] or
 * [n_masks][d_ff][d_model] per desc->w_layout.  packed_dev: mglu_packed_mask_bytes(desc)
 * bytes, fully overwritten. */
mglu_status mglu_pack_masks(const mglu_desc *desc, const uint8_t *masks_dev, void *packed_dev, void *stream);

/* ---- the per-token path (Eq. 3; Alg. 1) -------------------------------------------------- */

/* Bytes of scratch mglu_forward / mglu_forward_variant / mglu_ffn_forward need for this descriptor.
 * 0 wherever one launch covers the layer (its partial sums stay in registers and LDS).  With 9 to 16
 * masks and more than 32 tokens (16-bit types) the MFMA-tiled
 * kernel runs twice, 8 masks per launch, and hands the fp32 sum of the first launch's terms to the
 * second through the workspace: tokens * d_ff * 4 bytes.  0 also for an invalid descriptor. */
size_t mglu_workspace_bytes(const mglu_desc *desc);

/* out[tokens][d_ff] = MGLU_{n_masks}(x), Eq. 3 with g = Swish.
 *   x_dev            [tokens][d_model], desc->dtype
 *   W_packed_dev     from mglu_pack_weights with the same d_model, d_ff, dtype
 *   masks_packed_dev from mglu_pack_masks with the same d_model, d_ff, n_masks, dtype
 *   out_dev          [tokens][d_ff], desc->dtype, fully overwritten (rounded once, to
 *                    nearest-even, after the sum over masks)
 *   workspace_dev    at least mglu_workspace_bytes(desc) bytes, 16-byte aligned, may be NULL if that is 0;
 *                    contents need not be initialised and are not preserved; calls that may overlap on
 *                    the GPU (different streams) need a workspace each.
 * The result is deterministic: the same inputs give the same bits on every call. */
mglu_status mglu_forward(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                         const void *masks_packed_dev, void *out_dev,
                         void *workspace_dev, size_t workspace_bytes, void *stream);

/* Convenience form taking the unpacked W and byte masks (the layer as the paper states
 * it: x, W, {M_i}): packs both into the workspace, then runs mglu_forward.  For tests
 * and one-off calls; never the timed path.  Workspace: mglu_forward_bool_workspace_bytes(). */
size_t mglu_forward_bool_workspace_bytes(const mglu_desc *desc);
mglu_status mglu_forward_bool(const mglu_desc *desc, const void *x_dev, const void *W_dev,
                              const uint8_t *masks_dev, void *out_dev,
                              void *workspace_dev, size_t workspace_bytes, void *stream);

/* mglu_forward_bool for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, result and kernels as mglu_forward_bool, but the packed copies of W and the masks
 * are staged in a device array that is part of the library itself (MGLU_STATIC_SCRATCH_BYTES,
 * one copy on every GPU the library runs on, held until the process ends); the call allocates
 * and frees nothing.
 *   - Layers whose staging (mglu_forward_bool_workspace_bytes) exceeds MGLU_STATIC_SCRATCH_BYTES
 *     are rejected with MGLU_ERR_WORKSPACE before anything is enqueued.
 *   - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams,
 *     two threads) race on it.  Calls on one stream are ordered and safe; nothing of an earlier
 *     call's contents is relied on (both packed buffers are fully rewritten each time).
 *   - The first call on each device looks the array's address up once (no allocation; make that
 *     first call outside a graph capture). */
#define MGLU_STATIC_SCRATCH_BYTES (32u << 20)
mglu_status mglu_forward_bool_static(const mglu_desc *desc, const void *x_dev, const void *W_dev,
                                     const uint8_t *masks_dev, void *out_dev, void *stream);

/* Debug view of Alg. 1's accumulator z: the raw projections before the activation, fp32.
 *   t_dev [tokens][d_ff] = x W;  gate_dev, value_dev [n_masks][tokens][d_ff].
 * Any of the three may be NULL.  Same packed inputs and workspace rules as mglu_forward. */
mglu_status mglu_projections(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                             const void *masks_packed_dev, float *t_dev, float *gate_dev,
                             float *value_dev, void *workspace_dev, size_t workspace_bytes,
                             void *stream);

/* ---- variants from the paper's appendix, and the projection that follows the layer -------- */

/* Gate function g of Eq. 3 (appendix "Other Activation Functions": SwiMGLU, GeMGLU, ReMGLU). */
typedef enum {
    MGLU_GATE_SWISH = 0,   /* z * sigmoid(z), the main paper's choice */
    MGLU_GATE_GELU = 1,    /* z * Phi(z), exact Gaussian CDF */
    MGLU_GATE_RELU = 2     /* max(z, 0) */
} mglu_gate_fn;

/* Which branches see the masks (appendix "Partial Mask Ablation"); summed over masks as in Eq. 3. */
typedef enum {
    MGLU_MASK_BOTH = 0,        /* g(x (M_i*W))  * x ((1-M_i)*W)   Eq. 3 */
    MGLU_MASK_VALUE_ONLY = 1,  /* g(x W)        * x ((1-M_i)*W)   "No Gate Mask" (dense gate) */
    MGLU_MASK_GATE_ONLY = 2,   /* g(x (M_i*W))  * x W             "No Value Mask" (dense value) */
    MGLU_MASK_NONE = 3         /* g(x W)        * x W             "No Masks" */
} mglu_mask_use;

typedef struct {
    mglu_gate_fn gate;
    mglu_mask_use mask_use;
    /* Per-token route weights G(x)_i of the Top-K routed layer (appendix "Top-K Routing"):
     *   out = sum_i G(x)_i g(x (M_i*W)) * x ((1-M_i)*W).
     * dev, fp32 [tokens][n_masks], e.g. from mglu_route_topk; NULL means every weight is 1.
     * With at most 16 tokens (x resident in LDS) a mask whose weight is 0 for every token of the
     * call gets no sum at all -- no operand preparation, no MFMA; the selected masks share the
     * accumulators in compact order.  With more tokens every term is computed and then weighted.
     * The masks' bits stream from memory whatever the selection, so the saving is arithmetic only
     * (mglu_forward_routed with the planar mask format skips the bytes too). */
    const float *route_weights_dev;
} mglu_variant;

/* mglu_forward with the variations above; a NULL variant, or {SWISH, BOTH, NULL}, is mglu_forward. */
mglu_status mglu_forward_variant(const mglu_desc *desc, const mglu_variant *variant, const void *x_dev,
                                 const void *W_packed_dev, const void *masks_packed_dev, void *out_dev,
                                 void *workspace_dev, size_t workspace_bytes, void *stream);

/* Router of the Top-K routed layer: logits = x Wr, the k largest per token are kept (on equal
 * logits the lower mask index wins), softmax over the kept ones, 0 elsewhere.
 *   x_dev [tokens][d_model] and Wr_dev [d_model][n_masks] in desc->dtype; 1 <= k <= n_masks;
 *   weights_dev fp32 [tokens][n_masks], fully overwritten.  desc->d_ff is ignored. */
mglu_status mglu_route_topk(const mglu_desc *desc, const void *x_dev, const void *Wr_dev, int k,
                            float *weights_dev, void *stream);

/* ---- Top-K routed layer that reads only the selected masks (appendix "Top-K Routing") ------- */

/* The appendix notes that with Top-K routing only the K selected masked projections need be
 * evaluated, which cuts memory traffic as well as arithmetic.  The interleaved format of
 * mglu_pack_masks keeps the bits of all masks of an element side by side, so every mask's bits
 * stream whatever the selection.  This second, PLANAR format stores each mask's bit plane on its
 * own -- per column block and mask one contiguous run of 32-bit words, word = the 32 bits of that
 * mask for the 32 weight elements one lane holds in a chunk -- and mglu_forward_routed loads the
 * planes of the selected masks only: top-2 of 8 masks moves 16 + 2 instead of 16 + 8 bits per
 * weight element.  Exactly n_masks planes are stored (no rounding up). */
size_t mglu_packed_mask_bytes_planar(const mglu_desc *desc);
mglu_status mglu_pack_masks_planar(const mglu_desc *desc, const uint8_t *masks_dev, void *packed_dev, void *stream);

/* out = sum_i G(x)_i g(x (M_i*W)) * x ((1-M_i)*W) over the masks with a non-zero weight.
 *   masks_planar_dev   from mglu_pack_masks_planar
 *   route_weights_dev  fp32 [tokens][n_masks], e.g. from mglu_route_topk
 *   k                  how many weights per token may be non-zero (1 <= k <= n_masks): sizes the
 *                      kernel (accumulators for min(n_masks, k * tokens) masks, rounded up to 2, 4, 8
 *                      or 16).  The result is right for ANY weights: if more distinct masks turn out
 *                      to be selected than that, the kernel makes further passes over W for them.
 *   gate               the gate function g (MGLU_GATE_SWISH for the paper's routed SwiMGLU)
 * For at most 16 tokens whose rows of x fit the kernel's LDS budget (every decode shape of up to
 * ~28 K d_model at one token, 4096 at four); otherwise MGLU_ERR_UNSUPPORTED -- pack with
 * mglu_pack_masks and use mglu_forward_variant, which weights every mask's term, instead. */
mglu_status mglu_forward_routed(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                                const void *masks_planar_dev, const float *route_weights_dev, int k,
                                mglu_gate_fn gate, void *out_dev, void *stream);

/* Plain projection out = a W with the same packed weight format and kernels (no masks, no
 * activation): the output projection W_o in R^{d x h} that maps the layer's result back to the
 * hidden size (Method, after Eq. 1).  Here desc->d_model is the REDUCTION length (rows of the
 * unpacked W, = d_ff of the layer for W_o) and desc->d_ff the OUTPUT width (= d_model of the layer);
 * desc->n_masks is ignored.  a_dev [tokens][reduction], out_dev [tokens][output], desc->dtype. */
mglu_status mglu_linear_forward(const mglu_desc *desc, const void *a_dev, const void *W_packed_dev,
                                void *out_dev, void *workspace_dev, size_t workspace_bytes, void *stream);

/* The whole gated FFN block: y = MGLU(x) Wo, as two launches on `stream`.  desc describes the MGLU
 * layer; Wo_packed_dev comes from mglu_pack_weights with d_model and d_ff exchanged (Wo is
 * [d_ff][d_model] in the KN layout); hidden_dev [tokens][d_ff] is caller-owned scratch for the
 * intermediate representation; y_dev [tokens][d_model].  variant may be NULL. */
mglu_status mglu_ffn_forward(const mglu_desc *desc, const mglu_variant *variant, const void *x_dev,
                             const void *W_packed_dev, const void *masks_packed_dev,
                             const void *Wo_packed_dev, void *hidden_dev, void *y_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream);

/* ---- reference points for measurement ---------------------------------------------------- */

/* Two-matrix SwiGLU projection of the same shape (Eq. 1 with g = Swish), the paper's
 * "GLU" comparison: out = swish(x Wg) * (x Wv).  Wg_packed_dev and Wv_packed_dev each come
 * from mglu_pack_weights.  desc->n_masks is ignored.  Workspace as for mglu_forward. */
mglu_status swiglu_forward(const mglu_desc *desc, const void *x_dev, const void *Wg_packed_dev,
                           const void *Wv_packed_dev, void *out_dev,
                           void *workspace_dev, size_t workspace_bytes, void *stream);

/* Pure streaming read of `bytes` bytes (a multiple of 16) with the decode kernels'
 * access pattern; folds everything into sink_dev[0..255] (uint32, 1 KiB) so the reads
 * cannot be dropped.  Gives the read bandwidth this GPU actually reaches. */
mglu_status mglu_stream_read(const void *buf_dev, size_t bytes, uint32_t *sink_dev, void *stream);

/* ---- which kernel a call would run (host only; for tests and reports) ----------------------- */

/* The entry point being asked about. */
typedef enum {
    MGLU_CALL_FORWARD = 0,          /* mglu_forward, mglu_forward_bool */
    MGLU_CALL_FORWARD_VARIANT = 1,  /* mglu_forward_variant with any variation switched on */
    MGLU_CALL_PROJECTIONS = 2,      /* mglu_projections */
    MGLU_CALL_LINEAR = 3,           /* mglu_linear_forward */
    MGLU_CALL_SWIGLU = 4,           /* swiglu_forward */
    MGLU_CALL_FORWARD_ROUTED = 5    /* mglu_forward_routed */
} mglu_call;

/* Writes into buf (len bytes, always NUL-terminated) the name of the kernel instantiation that
 * `call` would launch for this descriptor -- kernel family and template arguments as in the
 * library's symbol table, e.g. "stream_resident_kernel<Bf16Traits, 8, 0, 2, false>" -- without
 * launching anything or touching a GPU.  The same checks as the call itself apply to the
 * descriptor; route_k is the `k` of mglu_forward_routed and ignored for every other call.  Lets a
 * test suite assert which code path a shape exercises, and that every instantiation the library
 * can select is covered by a parity test. */
mglu_status mglu_describe_plan(const mglu_desc *desc, mglu_call call, int route_k, char *buf, size_t len);

/* ---- errors -------------------------------------------------------------------------------- */
const char *mglu_last_error(void);              /* thread-local, never NULL */
const char *mglu_status_string(mglu_status s);  /* static text for a code */

#ifdef __cplusplus
}
#endif
#endif /* MGLU_H */
