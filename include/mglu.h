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
    MGLU_ERR_UNSUPPORTED = 2,  /* valid in principle, not built (e.g. n_masks > 8) */
    MGLU_ERR_WORKSPACE = 3,    /* workspace missing or smaller than the query says */
    MGLU_ERR_HIP = 4           /* the HIP runtime refused a launch */
} mglu_status;

/* Element type of x, W and out.  Accumulation is always fp32. */
typedef enum { MGLU_F32 = 0, MGLU_BF16 = 1 } mglu_dtype;

/* How the caller's UNPACKED weight matrix and mask planes are laid out (row-major):
 *   MGLU_W_KN: W [d_model][d_ff],  masks [n_masks][d_model][d_ff]   (the paper's math, W in R^{h x d})
 *   MGLU_W_NK: W [d_ff][d_model],  masks [n_masks][d_ff][d_model]   (the paper's kernel, A [M x N] with K contiguous)
 * Only the pack calls and mglu_forward_bool read it. */
typedef enum { MGLU_W_KN = 0, MGLU_W_NK = 1 } mglu_layout;

typedef struct {
    int32_t tokens;      /* T >= 1: rows of x and out (ignored by the pack calls) */
    int32_t d_model;     /* h >= 1: reduction length */
    int32_t d_ff;        /* d >= 1: output width */
    int32_t n_masks;     /* n_m in [1, 8] */
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
 * n_masks rounded up to 1, 2, 4 or 8 (the padding planes are all-zero, i.e. all-value,
 * and contribute exactly 0 to Eq. 3).  0 on a bad descriptor. */
size_t mglu_packed_mask_bytes(const mglu_desc *desc);

/* Packs n_masks planes of bytes (0 = value branch, non-zero = gate branch) into bit
 * planes in register-native order.  masks_dev: [n_masks][d_model][d_ff] or
 * [n_masks][d_ff][d_model] per desc->w_layout.  packed_dev: mglu_packed_mask_bytes(desc)
 * bytes, fully overwritten. */
mglu_status mglu_pack_masks(const mglu_desc *desc, const uint8_t *masks_dev, void *packed_dev, void *stream);

/* ---- the per-token path (Eq. 3; Alg. 1) -------------------------------------------------- */

/* Bytes of scratch mglu_forward needs for this descriptor (may be 0). */
size_t mglu_workspace_bytes(const mglu_desc *desc);

/* out[tokens][d_ff] = MGLU_{n_masks}(x), Eq. 3 with g = Swish.
 *   x_dev            [tokens][d_model], desc->dtype
 *   W_packed_dev     from mglu_pack_weights with the same d_model, d_ff, dtype
 *   masks_packed_dev from mglu_pack_masks with the same d_model, d_ff, n_masks, dtype
 *   out_dev          [tokens][d_ff], desc->dtype, fully overwritten (rounded once, to
 *                    nearest-even, after the sum over masks)
 *   workspace_dev    at least mglu_workspace_bytes(desc) bytes, may be NULL if that is 0.
 *                    Its contents need not be initialised, except that a workspace
 *                    used by the split reduction must have been zero-filled ONCE before
 *                    its first use (the kernels leave it zeroed again).
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

/* Debug view of Alg. 1's accumulator z: the raw projections before the activation, fp32.
 *   t_dev [tokens][d_ff] = x W;  gate_dev, value_dev [n_masks][tokens][d_ff].
 * Any of the three may be NULL.  Same packed inputs and workspace rules as mglu_forward. */
mglu_status mglu_projections(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                             const void *masks_packed_dev, float *t_dev, float *gate_dev,
                             float *value_dev, void *workspace_dev, size_t workspace_bytes,
                             void *stream);

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

/* ---- errors -------------------------------------------------------------------------------- */
const char *mglu_last_error(void);              /* thread-local, never NULL */
const char *mglu_status_string(mglu_status s);  /* static text for a code */

#ifdef __cplusplus
}
#endif
#endif /* MGLU_H */
