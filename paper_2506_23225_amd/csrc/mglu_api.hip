// C ABI of libmglu (declared in include/mglu.h): argument checks and kernel dispatch.
// No exception crosses the boundary; nothing here allocates device memory.
#include <stdarg.h>
#include <stdio.h>

#include "../../include/mglu.h"
#include "mglu_common.hpp"
#include "mglu_kernels.hpp"

#include <mutex>

namespace {

thread_local char g_error[512] = "";

mglu_status fail(mglu_status code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
    return code;
}

// the kernels' element kind of a descriptor's dtype (the two enums have the same values; spelled out
// so that neither header depends on the other)
int elem_of(const mglu_desc *d)
{
    return d->dtype == MGLU_F32 ? mglu::kElemF32 : d->dtype == MGLU_F16 ? mglu::kElemF16 : mglu::kElemBf16;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Shape part of the descriptor (everything but `tokens`).
mglu_status check_shape(const mglu_desc *d, bool need_masks)
{
    if (!d) return fail(MGLU_ERR_INVALID_ARG, "descriptor is NULL");
    if (d->dtype != MGLU_F32 && d->dtype != MGLU_BF16 && d->dtype != MGLU_F16)
        return fail(MGLU_ERR_INVALID_ARG, "dtype %d is none of MGLU_F32, MGLU_BF16, MGLU_F16", (int)d->dtype);
    if (d->w_layout != MGLU_W_KN && d->w_layout != MGLU_W_NK)
        return fail(MGLU_ERR_INVALID_ARG, "w_layout %d is neither MGLU_W_KN nor MGLU_W_NK", (int)d->w_layout);
    if (d->d_model < 1 || d->d_ff < 1)
        return fail(MGLU_ERR_INVALID_ARG, "d_model=%d and d_ff=%d must be >= 1", d->d_model, d->d_ff);
    if (need_masks) {
        if (d->n_masks < 1) return fail(MGLU_ERR_INVALID_ARG, "n_masks=%d must be >= 1", d->n_masks);
        if (d->n_masks > mglu::kMaxMasks)
            return fail(MGLU_ERR_UNSUPPORTED, "n_masks=%d: at most %d masks are supported", d->n_masks, mglu::kMaxMasks);
    }
    const long nb = mglu::ceil_div(d->d_ff, mglu::kColBlock), nc = mglu::ceil_div(d->d_model, mglu::kChunkK);
    if (nb > 0x7fffffffL / 64 || nb * nc > 0x7fffffffL / 8)
        return fail(MGLU_ERR_UNSUPPORTED, "d_model=%d x d_ff=%d is too large", d->d_model, d->d_ff);
    return MGLU_OK;
}

mglu_status check_forward(const mglu_desc *d, bool need_masks)
{
    mglu_status s = check_shape(d, need_masks);
    if (s != MGLU_OK) return s;
    if (d->tokens < 1) return fail(MGLU_ERR_INVALID_ARG, "tokens=%d must be >= 1", d->tokens);
    const int lane_k = d->dtype == MGLU_F32 ? 4 : 8;
    if (d->d_model % lane_k != 0)
        return fail(MGLU_ERR_UNSUPPORTED, "d_model=%d must be a multiple of %d so that rows of x stay 16-byte aligned",
                    d->d_model, lane_k);
    if ((long)d->tokens * d->d_ff > 0x7fffffff00L)
        return fail(MGLU_ERR_UNSUPPORTED, "tokens=%d x d_ff=%d is too large", d->tokens, d->d_ff);
    if (d->tokens > 16 * 65535)   // token groups ride on gridDim.y
        return fail(MGLU_ERR_UNSUPPORTED, "tokens=%d: at most %d tokens per call", d->tokens, 16 * 65535);
    return MGLU_OK;
}

mglu_status check_ptr(const void *p, const char *name)
{
    if (!p) return fail(MGLU_ERR_INVALID_ARG, "%s is NULL", name);
    if (!aligned16(p)) return fail(MGLU_ERR_INVALID_ARG, "%s is not 16-byte aligned", name);
    return MGLU_OK;
}

mglu_status hip_result(hipError_t e, const char *what)
{
    if (e == hipSuccess) return MGLU_OK;
    return fail(MGLU_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

mglu::StreamParams stream_params(const mglu_desc *d)
{
    mglu::StreamParams p = {};
    p.T = d->tokens;
    p.h = d->d_model;
    p.d = d->d_ff;
    p.n_masks = d->n_masks;
    p.NB = (int)mglu::ceil_div(d->d_ff, mglu::kColBlock);
    p.NC = (int)mglu::ceil_div(d->d_model, mglu::kChunkK);
    return p;
}

// Token counts the streaming kernels cover in one pass over W (64 with one or two masks, 32 with up to
// eight, 16 beyond) stay on them: there the layer is bound by streaming W.  Above that the 16-bit types
// go to the MFMA-tiled kernel, whose small tile shapes fill the chip from a few dozen tokens on.
bool use_tiled_kernel(const mglu_desc *d, int n_masks)
{
    if (d->dtype == MGLU_F32) return false;
    return d->tokens > 16 * mglu::stream_max_token_blocks(mglu::round_up_masks(n_masks), elem_of(d));
}

mglu::PrefillParams prefill_params(const mglu_desc *d)
{
    mglu::PrefillParams p = {};
    p.T = d->tokens;
    p.h = d->d_model;
    p.d = d->d_ff;
    p.n_masks = d->n_masks;
    p.NB = (int)mglu::ceil_div(d->d_ff, mglu::kColBlock);
    p.NC = (int)mglu::ceil_div(d->d_model, mglu::kChunkK);
    return p;
}

mglu::PackParams pack_params(const mglu_desc *d, const void *src, void *dst)
{
    mglu::PackParams p = {};
    p.src = src;
    p.dst = dst;
    p.h = d->d_model;
    p.d = d->d_ff;
    p.n_masks = d->n_masks;
    p.NB = (int)mglu::ceil_div(d->d_ff, mglu::kColBlock);
    p.NC = (int)mglu::ceil_div(d->d_model, mglu::kChunkK);
    p.nk = d->w_layout == MGLU_W_NK;
    return p;
}

#define MGLU_TRY(expr)                      \
    do {                                    \
        mglu_status s_ = (expr);            \
        if (s_ != MGLU_OK) return s_;       \
    } while (0)


// Everything a launch reads and writes besides the descriptor; unused members stay null / 0.
struct Operands {
    const void *x, *w, *w2;
    const uint32_t *m;
    void *out;
    float *proj_t, *proj_gate, *proj_value;
    int gate_fn, mask_use;
    const float *route;
    void *workspace;
    size_t workspace_bytes;
};

// fp32 [tokens][d_ff] for the MFMA-tiled kernel with more than 8 masks (two launches of 8 masks)
size_t layer_workspace_bytes(const mglu_desc *d)
{
    if (!use_tiled_kernel(d, d->n_masks) || !mglu::prefill_two_launches(d->n_masks, d->tokens)) return 0;
    return (size_t)d->tokens * d->d_ff * sizeof(float);
}

// The one place that picks the kernel family for a call: `mode` is a mglu::Mode.  With `describe` set
// nothing is launched and the chosen kernel instantiation is written there instead.
mglu_status run_layer(const mglu_desc *d, int mode, const Operands &o, void *stream, const char *what,
                      char *describe = nullptr, size_t describe_len = 0)
{
    const int n_masks = (mode == mglu::kModeLinear || mode == mglu::kModeSwiglu) ? 1 : d->n_masks;
    if (mode != mglu::kModeProjections && use_tiled_kernel(d, n_masks)) {
        mglu::PrefillParams pp = prefill_params(d);
        pp.x = o.x; pp.w = o.w; pp.w2 = o.w2; pp.m = o.m; pp.out = o.out;
        pp.gate_fn = o.gate_fn; pp.mask_use = o.mask_use; pp.route = o.route;
        pp.describe = describe; pp.describe_len = describe_len;
        if (mode == mglu::kModeMglu || mode == mglu::kModeMgluVariant) {
            const size_t need = layer_workspace_bytes(d);
            if (describe) {
                pp.workspace = need ? reinterpret_cast<float *>(uintptr_t(256)) : nullptr;   // never dereferenced
            } else if (need) {
                if (!o.workspace || o.workspace_bytes < need)
                    return fail(MGLU_ERR_WORKSPACE, "workspace has %zu bytes, this layer needs %zu (mglu_workspace_bytes)",
                                o.workspace ? o.workspace_bytes : (size_t)0, need);
                MGLU_TRY(check_ptr(o.workspace, "workspace_dev"));
                pp.workspace = static_cast<float *>(o.workspace);
            }
        }
        return hip_result(mglu::launch_prefill(pp, elem_of(d), mode, static_cast<hipStream_t>(stream)), what);
    }
    mglu::StreamParams p = stream_params(d);
    p.x = o.x; p.w = o.w; p.w2 = o.w2; p.m = o.m; p.out = o.out;
    p.proj_t = o.proj_t; p.proj_gate = o.proj_gate; p.proj_value = o.proj_value;
    p.gate_fn = o.gate_fn; p.mask_use = o.mask_use; p.route = o.route;
    p.describe = describe; p.describe_len = describe_len;
    return hip_result(mglu::launch_stream(p, elem_of(d), mode, static_cast<hipStream_t>(stream)), what);
}

// Shape part of a routed call, checked: k, the gate, and whether the routed kernel covers the shape.
mglu_status routed_params(const mglu_desc *d, int k, int gate, mglu::RoutedParams *rp)
{
    if (k < 1 || k > d->n_masks) return fail(MGLU_ERR_INVALID_ARG, "k=%d must be in [1, n_masks=%d]", k, d->n_masks);
    if (gate < MGLU_GATE_SWISH || gate > MGLU_GATE_RELU) return fail(MGLU_ERR_INVALID_ARG, "gate %d is not a mglu_gate_fn", gate);
    rp->T = d->tokens;
    rp->h = d->d_model;
    rp->d = d->d_ff;
    rp->n_masks = d->n_masks;
    rp->NB = (int)mglu::ceil_div(d->d_ff, mglu::kColBlock);
    rp->NC = (int)mglu::ceil_div(d->d_model, mglu::kChunkK);
    rp->gate_fn = gate;
    rp->k = k;
    if (!mglu::routed_supported(*rp, elem_of(d)))
        return fail(MGLU_ERR_UNSUPPORTED,
                    "mglu_forward_routed covers at most 16 tokens whose rows of x fit its LDS budget (tokens=%d, d_model=%d): "
                    "pack with mglu_pack_masks and use mglu_forward_variant instead", d->tokens, d->d_model);
    return MGLU_OK;
}

mglu_status check_bool_inputs(const void *x_dev, const void *W_dev, const uint8_t *masks_dev, const void *out_dev)
{
    MGLU_TRY(check_ptr(x_dev, "x_dev"));
    MGLU_TRY(check_ptr(W_dev, "W_dev"));
    MGLU_TRY(check_ptr(masks_dev, "masks_dev"));
    return check_ptr(out_dev, "out_dev");
}

// ---- device memory that belongs to the library: staging for mglu_forward_bool_static ----
// One array per GPU (every device the code object is loaded on holds its own copy at its own
// address, until the process ends).  In host code the array's name is only a handle for the
// symbol look-up below; what kernels and the pack calls get is the device address it returns.
__device__ __align__(256) unsigned char scratch[MGLU_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_lock;
char *g_scratch_ptr[kMaxDevices] = {};

// The current device's copy of the array; looked up once per device, with that device current.
mglu_status static_scratch(char **out)
{
    int dev = -1;
    MGLU_TRY(hip_result(hipGetDevice(&dev), "hipGetDevice"));
    if (dev < 0 || dev >= kMaxDevices) return fail(MGLU_ERR_UNSUPPORTED, "device ordinal %d is beyond %d", dev, kMaxDevices);
    std::lock_guard<std::mutex> guard(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        MGLU_TRY(hip_result(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)"));
        if (!ptr || (reinterpret_cast<uintptr_t>(ptr) & 255u))
            return fail(MGLU_ERR_HIP, "the static scratch array has no usable device address");
        g_scratch_ptr[dev] = static_cast<char *>(ptr);
    }
    *out = g_scratch_ptr[dev];
    return MGLU_OK;
}

}  // namespace

extern "C" {

int mglu_format_version(void) { return 5; }

size_t mglu_packed_weight_bytes(const mglu_desc *desc)
{
    if (check_shape(desc, false) != MGLU_OK) return 0;
    const size_t nb = mglu::ceil_div(desc->d_ff, mglu::kColBlock), nc = mglu::ceil_div(desc->d_model, mglu::kChunkK);
    return nb * nc * mglu::kColBlock * mglu::kChunkK * (desc->dtype == MGLU_F32 ? 4 : 2);
}

size_t mglu_packed_mask_bytes(const mglu_desc *desc)
{
    if (check_shape(desc, true) != MGLU_OK) return 0;
    const size_t nb = mglu::ceil_div(desc->d_ff, mglu::kColBlock), nc = mglu::ceil_div(desc->d_model, mglu::kChunkK);
    return nb * nc * mglu::kWave * mglu::round_up_masks(desc->n_masks) * sizeof(uint32_t);
}

mglu_status mglu_pack_weights(const mglu_desc *desc, const void *W_dev, void *packed_dev, void *stream)
{
    MGLU_TRY(check_shape(desc, false));
    MGLU_TRY(check_ptr(W_dev, "W_dev"));
    MGLU_TRY(check_ptr(packed_dev, "packed_dev"));
    return hip_result(mglu::launch_pack_weights(pack_params(desc, W_dev, packed_dev), elem_of(desc),
                                                static_cast<hipStream_t>(stream)),
                      "mglu_pack_weights launch");
}

mglu_status mglu_pack_masks(const mglu_desc *desc, const uint8_t *masks_dev, void *packed_dev, void *stream)
{
    MGLU_TRY(check_shape(desc, true));
    MGLU_TRY(check_ptr(masks_dev, "masks_dev"));
    MGLU_TRY(check_ptr(packed_dev, "packed_dev"));
    return hip_result(mglu::launch_pack_masks(pack_params(desc, masks_dev, packed_dev), elem_of(desc),
                                              static_cast<hipStream_t>(stream)),
                      "mglu_pack_masks launch");
}

size_t mglu_packed_mask_bytes_planar(const mglu_desc *desc)
{
    if (check_shape(desc, true) != MGLU_OK) return 0;
    const size_t nb = mglu::ceil_div(desc->d_ff, mglu::kColBlock), nc = mglu::ceil_div(desc->d_model, mglu::kChunkK);
    return nb * nc * mglu::kWave * (size_t)desc->n_masks * sizeof(uint32_t);
}

mglu_status mglu_pack_masks_planar(const mglu_desc *desc, const uint8_t *masks_dev, void *packed_dev, void *stream)
{
    MGLU_TRY(check_shape(desc, true));
    MGLU_TRY(check_ptr(masks_dev, "masks_dev"));
    MGLU_TRY(check_ptr(packed_dev, "packed_dev"));
    return hip_result(mglu::launch_pack_masks_planar(pack_params(desc, masks_dev, packed_dev), elem_of(desc),
                                                     static_cast<hipStream_t>(stream)),
                      "mglu_pack_masks_planar launch");
}

size_t mglu_workspace_bytes(const mglu_desc *desc)
{
    if (check_shape(desc, true) != MGLU_OK) return 0;
    return layer_workspace_bytes(desc);
}

mglu_status mglu_forward_variant(const mglu_desc *desc, const mglu_variant *variant, const void *x_dev,
                                 const void *W_packed_dev, const void *masks_packed_dev, void *out_dev,
                                 void *workspace_dev, size_t workspace_bytes, void *stream)
{
    MGLU_TRY(check_forward(desc, true));
    MGLU_TRY(check_ptr(x_dev, "x_dev"));
    MGLU_TRY(check_ptr(W_packed_dev, "W_packed_dev"));
    MGLU_TRY(check_ptr(masks_packed_dev, "masks_packed_dev"));
    MGLU_TRY(check_ptr(out_dev, "out_dev"));
    int gate_fn = 0, mask_use = 0;
    const float *route = nullptr;
    if (variant) {
        if (variant->gate < MGLU_GATE_SWISH || variant->gate > MGLU_GATE_RELU)
            return fail(MGLU_ERR_INVALID_ARG, "variant->gate %d is not a mglu_gate_fn", (int)variant->gate);
        if (variant->mask_use < MGLU_MASK_BOTH || variant->mask_use > MGLU_MASK_NONE)
            return fail(MGLU_ERR_INVALID_ARG, "variant->mask_use %d is not a mglu_mask_use", (int)variant->mask_use);
        if (variant->route_weights_dev && (reinterpret_cast<uintptr_t>(variant->route_weights_dev) & 3u))
            return fail(MGLU_ERR_INVALID_ARG, "variant->route_weights_dev is not 4-byte aligned");
        gate_fn = (int)variant->gate;
        mask_use = (int)variant->mask_use;
        route = variant->route_weights_dev;
    }
    // the main form (Swish, both branches masked, no route weights) runs the kernels without the run-time choices
    const int mode = (gate_fn != 0 || mask_use != 0 || route) ? mglu::kModeMgluVariant : mglu::kModeMglu;
    Operands o = {};
    o.x = x_dev; o.w = W_packed_dev; o.m = static_cast<const uint32_t *>(masks_packed_dev); o.out = out_dev;
    o.gate_fn = gate_fn; o.mask_use = mask_use; o.route = route;
    o.workspace = workspace_dev; o.workspace_bytes = workspace_bytes;
    return run_layer(desc, mode, o, stream, "mglu_forward launch");
}

mglu_status mglu_forward(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                         const void *masks_packed_dev, void *out_dev, void *workspace_dev,
                         size_t workspace_bytes, void *stream)
{
    return mglu_forward_variant(desc, nullptr, x_dev, W_packed_dev, masks_packed_dev, out_dev, workspace_dev,
                                workspace_bytes, stream);
}

mglu_status mglu_forward_routed(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                                const void *masks_planar_dev, const float *route_weights_dev, int k,
                                mglu_gate_fn gate, void *out_dev, void *stream)
{
    MGLU_TRY(check_forward(desc, true));
    MGLU_TRY(check_ptr(x_dev, "x_dev"));
    MGLU_TRY(check_ptr(W_packed_dev, "W_packed_dev"));
    MGLU_TRY(check_ptr(masks_planar_dev, "masks_planar_dev"));
    MGLU_TRY(check_ptr(out_dev, "out_dev"));
    if (!route_weights_dev || (reinterpret_cast<uintptr_t>(route_weights_dev) & 3u))
        return fail(MGLU_ERR_INVALID_ARG, "route_weights_dev is NULL or not 4-byte aligned");
    mglu::RoutedParams rp = {};
    MGLU_TRY(routed_params(desc, k, (int)gate, &rp));
    rp.x = x_dev;
    rp.w = W_packed_dev;
    rp.m = static_cast<const uint32_t *>(masks_planar_dev);
    rp.route = route_weights_dev;
    rp.out = out_dev;
    return hip_result(mglu::launch_routed(rp, elem_of(desc), static_cast<hipStream_t>(stream)),
                      "mglu_forward_routed launch");
}

mglu_status mglu_route_topk(const mglu_desc *desc, const void *x_dev, const void *Wr_dev, int k,
                            float *weights_dev, void *stream)
{
    if (!desc) return fail(MGLU_ERR_INVALID_ARG, "descriptor is NULL");
    if (desc->dtype != MGLU_F32 && desc->dtype != MGLU_BF16 && desc->dtype != MGLU_F16)
        return fail(MGLU_ERR_INVALID_ARG, "dtype %d is none of MGLU_F32, MGLU_BF16, MGLU_F16", (int)desc->dtype);
    if (desc->tokens < 1 || desc->d_model < 1)
        return fail(MGLU_ERR_INVALID_ARG, "tokens=%d and d_model=%d must be >= 1", desc->tokens, desc->d_model);
    if (desc->n_masks < 1) return fail(MGLU_ERR_INVALID_ARG, "n_masks=%d must be >= 1", desc->n_masks);
    if (desc->n_masks > mglu::kMaxMasks)
        return fail(MGLU_ERR_UNSUPPORTED, "n_masks=%d: at most %d masks are supported", desc->n_masks, mglu::kMaxMasks);
    if (k < 1 || k > desc->n_masks) return fail(MGLU_ERR_INVALID_ARG, "k=%d must be in [1, n_masks=%d]", k, desc->n_masks);
    MGLU_TRY(check_ptr(x_dev, "x_dev"));
    MGLU_TRY(check_ptr(Wr_dev, "Wr_dev"));
    MGLU_TRY(check_ptr(weights_dev, "weights_dev"));
    mglu::RouteParams rp = {};
    rp.x = x_dev;
    rp.wr = Wr_dev;
    rp.weights = weights_dev;
    rp.T = desc->tokens;
    rp.h = desc->d_model;
    rp.n_masks = desc->n_masks;
    rp.k = k;
    return hip_result(mglu::launch_route_topk(rp, elem_of(desc), static_cast<hipStream_t>(stream)),
                      "mglu_route_topk launch");
}

mglu_status mglu_linear_forward(const mglu_desc *desc, const void *a_dev, const void *W_packed_dev,
                                void *out_dev, void *workspace_dev, size_t workspace_bytes, void *stream)
{
    MGLU_TRY(check_forward(desc, false));
    MGLU_TRY(check_ptr(a_dev, "a_dev"));
    MGLU_TRY(check_ptr(W_packed_dev, "W_packed_dev"));
    MGLU_TRY(check_ptr(out_dev, "out_dev"));
    (void)workspace_dev;
    (void)workspace_bytes;
    Operands o = {};
    o.x = a_dev; o.w = W_packed_dev; o.out = out_dev;
    return run_layer(desc, mglu::kModeLinear, o, stream, "mglu_linear_forward launch");
}

mglu_status mglu_ffn_forward(const mglu_desc *desc, const mglu_variant *variant, const void *x_dev,
                             const void *W_packed_dev, const void *masks_packed_dev,
                             const void *Wo_packed_dev, void *hidden_dev, void *y_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream)
{
    MGLU_TRY(check_forward(desc, true));
    MGLU_TRY(check_ptr(hidden_dev, "hidden_dev"));
    MGLU_TRY(check_ptr(Wo_packed_dev, "Wo_packed_dev"));
    MGLU_TRY(check_ptr(y_dev, "y_dev"));
    mglu_desc down = *desc;        // the output projection reduces over d_ff and produces d_model columns
    down.d_model = desc->d_ff;
    down.d_ff = desc->d_model;
    MGLU_TRY(check_forward(&down, false));
    MGLU_TRY(mglu_forward_variant(desc, variant, x_dev, W_packed_dev, masks_packed_dev, hidden_dev, workspace_dev,
                                  workspace_bytes, stream));
    return mglu_linear_forward(&down, hidden_dev, Wo_packed_dev, y_dev, workspace_dev, workspace_bytes, stream);
}

// Packs W and the masks into `ws` (arguments already checked, `ws` large enough), then runs the layer on them.
static mglu_status pack_and_forward(const mglu_desc *desc, const void *x_dev, const void *W_dev,
                                    const uint8_t *masks_dev, void *out_dev, char *ws, size_t ws_bytes, void *stream)
{
    void *wp = ws;
    void *mp = ws + align_up(mglu_packed_weight_bytes(desc), 256);
    char *fw = static_cast<char *>(mp) + align_up(mglu_packed_mask_bytes(desc), 256);
    MGLU_TRY(mglu_pack_weights(desc, W_dev, wp, stream));
    MGLU_TRY(mglu_pack_masks(desc, masks_dev, mp, stream));
    return mglu_forward(desc, x_dev, wp, mp, out_dev, fw, ws_bytes - (size_t)(fw - ws), stream);
}

size_t mglu_forward_bool_workspace_bytes(const mglu_desc *desc)
{
    const size_t w = mglu_packed_weight_bytes(desc), m = mglu_packed_mask_bytes(desc);
    if (w == 0 || m == 0) return 0;
    return align_up(w, 256) + align_up(m, 256) + align_up(mglu_workspace_bytes(desc), 256);
}

mglu_status mglu_forward_bool(const mglu_desc *desc, const void *x_dev, const void *W_dev,
                              const uint8_t *masks_dev, void *out_dev, void *workspace_dev,
                              size_t workspace_bytes, void *stream)
{
    MGLU_TRY(check_forward(desc, true));
    MGLU_TRY(check_bool_inputs(x_dev, W_dev, masks_dev, out_dev));
    MGLU_TRY(check_ptr(workspace_dev, "workspace_dev"));
    const size_t need = mglu_forward_bool_workspace_bytes(desc);
    if (workspace_bytes < need)
        return fail(MGLU_ERR_WORKSPACE, "workspace has %zu bytes, mglu_forward_bool needs %zu", workspace_bytes, need);
    return pack_and_forward(desc, x_dev, W_dev, masks_dev, out_dev, static_cast<char *>(workspace_dev),
                            workspace_bytes, stream);
}

mglu_status mglu_forward_bool_static(const mglu_desc *desc, const void *x_dev, const void *W_dev,
                                     const uint8_t *masks_dev, void *out_dev, void *stream)
{
    MGLU_TRY(check_forward(desc, true));
    MGLU_TRY(check_bool_inputs(x_dev, W_dev, masks_dev, out_dev));
    const size_t need = mglu_forward_bool_workspace_bytes(desc);
    if (need > (size_t)MGLU_STATIC_SCRATCH_BYTES)
        return fail(MGLU_ERR_WORKSPACE,
                    "mglu_forward_bool_static: d_model=%d x d_ff=%d with %d masks needs %zu bytes of staging, the "
                    "library's static scratch holds %zu; use mglu_forward_bool with a workspace of your own",
                    desc->d_model, desc->d_ff, desc->n_masks, need, (size_t)MGLU_STATIC_SCRATCH_BYTES);
    char *ws = nullptr;
    MGLU_TRY(static_scratch(&ws));
    return pack_and_forward(desc, x_dev, W_dev, masks_dev, out_dev, ws, (size_t)MGLU_STATIC_SCRATCH_BYTES, stream);
}

mglu_status mglu_projections(const mglu_desc *desc, const void *x_dev, const void *W_packed_dev,
                             const void *masks_packed_dev, float *t_dev, float *gate_dev, float *value_dev,
                             void *workspace_dev, size_t workspace_bytes, void *stream)
{
    MGLU_TRY(check_forward(desc, true));
    MGLU_TRY(check_ptr(x_dev, "x_dev"));
    MGLU_TRY(check_ptr(W_packed_dev, "W_packed_dev"));
    MGLU_TRY(check_ptr(masks_packed_dev, "masks_packed_dev"));
    if (t_dev) MGLU_TRY(check_ptr(t_dev, "t_dev"));
    if (gate_dev) MGLU_TRY(check_ptr(gate_dev, "gate_dev"));
    if (value_dev) MGLU_TRY(check_ptr(value_dev, "value_dev"));
    (void)workspace_dev;
    (void)workspace_bytes;
    Operands o = {};
    o.x = x_dev; o.w = W_packed_dev; o.m = static_cast<const uint32_t *>(masks_packed_dev);
    o.proj_t = t_dev; o.proj_gate = gate_dev; o.proj_value = value_dev;
    return run_layer(desc, mglu::kModeProjections, o, stream, "mglu_projections launch");
}

mglu_status swiglu_forward(const mglu_desc *desc, const void *x_dev, const void *Wg_packed_dev,
                           const void *Wv_packed_dev, void *out_dev, void *workspace_dev,
                           size_t workspace_bytes, void *stream)
{
    MGLU_TRY(check_forward(desc, false));
    MGLU_TRY(check_ptr(x_dev, "x_dev"));
    MGLU_TRY(check_ptr(Wg_packed_dev, "Wg_packed_dev"));
    MGLU_TRY(check_ptr(Wv_packed_dev, "Wv_packed_dev"));
    MGLU_TRY(check_ptr(out_dev, "out_dev"));
    (void)workspace_dev;
    (void)workspace_bytes;
    Operands o = {};
    o.x = x_dev; o.w = Wg_packed_dev; o.w2 = Wv_packed_dev; o.out = out_dev;
    return run_layer(desc, mglu::kModeSwiglu, o, stream, "swiglu_forward launch");
}

mglu_status mglu_describe_plan(const mglu_desc *desc, mglu_call call, int route_k, char *buf, size_t len)
{
    if (!buf || len == 0) return fail(MGLU_ERR_INVALID_ARG, "buf is NULL or has no room");
    buf[0] = '\0';
    if (call == MGLU_CALL_FORWARD_ROUTED) {
        MGLU_TRY(check_forward(desc, true));
        mglu::RoutedParams rp = {};
        MGLU_TRY(routed_params(desc, route_k, MGLU_GATE_SWISH, &rp));
        rp.describe = buf;
        rp.describe_len = len;
        return hip_result(mglu::launch_routed(rp, elem_of(desc), nullptr), "mglu_describe_plan");
    }
    int mode;
    switch (call) {
    case MGLU_CALL_FORWARD: mode = mglu::kModeMglu; break;
    case MGLU_CALL_FORWARD_VARIANT: mode = mglu::kModeMgluVariant; break;
    case MGLU_CALL_PROJECTIONS: mode = mglu::kModeProjections; break;
    case MGLU_CALL_LINEAR: mode = mglu::kModeLinear; break;
    case MGLU_CALL_SWIGLU: mode = mglu::kModeSwiglu; break;
    default: return fail(MGLU_ERR_INVALID_ARG, "call %d is not a mglu_call", (int)call);
    }
    MGLU_TRY(check_forward(desc, mode != mglu::kModeLinear && mode != mglu::kModeSwiglu));
    return run_layer(desc, mode, Operands{}, nullptr, "mglu_describe_plan", buf, len);
}

mglu_status mglu_stream_read(const void *buf_dev, size_t bytes, uint32_t *sink_dev, void *stream)
{
    MGLU_TRY(check_ptr(buf_dev, "buf_dev"));
    MGLU_TRY(check_ptr(sink_dev, "sink_dev"));
    if (bytes == 0 || bytes % 16 != 0)
        return fail(MGLU_ERR_INVALID_ARG, "bytes=%zu must be a positive multiple of 16", bytes);
    return hip_result(mglu::launch_stream_read(buf_dev, bytes, sink_dev, static_cast<hipStream_t>(stream)),
                      "mglu_stream_read launch");
}

const char *mglu_last_error(void) { return g_error; }

const char *mglu_status_string(mglu_status s)
{
    switch (s) {
    case MGLU_OK: return "ok";
    case MGLU_ERR_INVALID_ARG: return "invalid argument";
    case MGLU_ERR_UNSUPPORTED: return "unsupported";
    case MGLU_ERR_WORKSPACE: return "workspace too small";
    case MGLU_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

}  // extern "C"
