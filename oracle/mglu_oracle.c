/*
 * MGLU forward oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A slow, plain fp64 CPU statement of what the Masked Gated Linear Unit
 * computes.  Only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it; the GPU library shares no source, header, table or helper
 * with this file and never routes through it.
 *
 * What is computed (paper, Method section):
 *   Eq. 2 (single mask):  MGLU_1(x)  = g( x (M (.) W) ) (.) ( x (Mbar (.) W) ),  Mbar = 1 - M
 *   Eq. 3 (MoEG):         MGLU_nm(x) = sum_{i=1..n_m} g( x (M_i (.) W) ) (.) ( x (Mbar_i (.) W) )
 *   g = Swish, g(z) = z * sigmoid(z)  (Related Work, "Choices of Activation Functions")
 *   Eq. 1 (GLU):          GLU(x)     = g( x W_g ) (.) ( x W_v )
 * No bias (footnote to Eq. 1).  A batch of token rows is that map applied to
 * each row on its own.
 *
 * How: for every mask i the two masked matrices M_i (.) W and Mbar_i (.) W are
 * materialised and each is multiplied by x with a plain matrix product, the
 * way the paper's training-time layer (appendix "PyTorch Implementation of
 * MGLU") forms its two projections.  Nothing of the fast kernel's design is
 * used here: no bit packing, no complement trick (value is NOT formed as
 * xW - gate), no split of the reduction dimension.
 *
 * Readings of the paper taken here:
 *   - Swish has beta = 1.
 *   - A mask bit of 1 sends the weight element to the gate branch (the one the
 *     activation is applied to); a 0 sends it to the value branch (Eq. 2;
 *     Alg. 1 adds v to s_i when the bit is set and writes s_i as the gate row).
 *   - The mixture is a plain sum: no 1/n_m, no router.
 *   - W is indexed logically W[k][j], k in [0,h) the reduction (hidden) index,
 *     j in [0,d) the output (intermediate) index; masks share that indexing.
 *
 * Layouts (all row-major, all host memory, caller-owned):
 *   x     double  [T][h]
 *   W     double  [h][d]
 *   M     uint8_t [n_m][h][d], every byte 0 or 1
 *   out   double  [T][d]
 *   gate, value (optional, may be NULL)  double [n_m][T][d]
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Swish with beta = 1:  z * sigmoid(z) = z / (1 + exp(-z)). */
static double swish(double z) { return z / (1.0 + exp(-z)); }

/* y[T][d] = x[T][h] * A[h][d], every output summed over k = 0..h-1 in
 * ascending order.  Threads take disjoint column ranges; within a range the
 * loops run token, then k, then column, so each A row segment is read once. */
static void matmul(const double *x, const double *A, double *y, long T, long h, long d)
{
    const long col_chunk = 256;
    const long n_chunks = (d + col_chunk - 1) / col_chunk;
#pragma omp parallel for schedule(static)
    for (long c = 0; c < n_chunks; ++c) {
        const long j0 = c * col_chunk;
        const long j1 = (j0 + col_chunk < d) ? j0 + col_chunk : d;
        for (long tau = 0; tau < T; ++tau) {
            double *yrow = y + tau * d;
            for (long j = j0; j < j1; ++j) yrow[j] = 0.0;
            for (long k = 0; k < h; ++k) {
                const double xv = x[tau * h + k];
                const double *arow = A + k * d;
                for (long j = j0; j < j1; ++j) yrow[j] += xv * arow[j];
            }
        }
    }
}

/* Eq. 3.  Returns 0 on success, 1 on a bad argument, 2 if memory ran out. */
int mglu_oracle_forward(const double *x, const double *W, const uint8_t *M,
                        long T, long h, long d, long n_m,
                        double *out, double *gate_out, double *value_out)
{
    if (!x || !W || !M || !out || T < 0 || h < 0 || d < 0 || n_m < 0) return 1;
    const long hd = h * d, Td = T * d;
    for (long e = 0; e < Td; ++e) out[e] = 0.0;
    if (Td == 0 || n_m == 0) return 0;

    double *Wg = (double *)malloc(sizeof(double) * (size_t)(hd > 0 ? hd : 1));
    double *Wv = (double *)malloc(sizeof(double) * (size_t)(hd > 0 ? hd : 1));
    double *gate = (double *)malloc(sizeof(double) * (size_t)Td);
    double *value = (double *)malloc(sizeof(double) * (size_t)Td);
    if (!Wg || !Wv || !gate || !value) {
        free(Wg); free(Wv); free(gate); free(value);
        return 2;
    }

    for (long i = 0; i < n_m; ++i) {
        const uint8_t *Mi = M + i * hd;
        /* gate matrix M_i (.) W and value matrix (1 - M_i) (.) W */
#pragma omp parallel for schedule(static)
        for (long e = 0; e < hd; ++e) {
            const double m = (double)(Mi[e] != 0);
            Wg[e] = m * W[e];
            Wv[e] = (1.0 - m) * W[e];
        }
        matmul(x, Wg, gate, T, h, d);
        matmul(x, Wv, value, T, h, d);
        for (long e = 0; e < Td; ++e) out[e] += swish(gate[e]) * value[e];
        if (gate_out) memcpy(gate_out + i * Td, gate, sizeof(double) * (size_t)Td);
        if (value_out) memcpy(value_out + i * Td, value, sizeof(double) * (size_t)Td);
    }
    free(Wg); free(Wv); free(gate); free(value);
    return 0;
}

/* Eq. 1 with g = Swish: the two-matrix SwiGLU projection.  Wg, Wv double [h][d]. */
int swiglu_oracle_forward(const double *x, const double *Wg, const double *Wv,
                          long T, long h, long d, double *out)
{
    if (!x || !Wg || !Wv || !out || T < 0 || h < 0 || d < 0) return 1;
    const long Td = T * d;
    if (Td == 0) return 0;
    double *gate = (double *)malloc(sizeof(double) * (size_t)Td);
    double *value = (double *)malloc(sizeof(double) * (size_t)Td);
    if (!gate || !value) { free(gate); free(value); return 2; }
    matmul(x, Wg, gate, T, h, d);
    matmul(x, Wv, value, T, h, d);
    for (long e = 0; e < Td; ++e) out[e] = swish(gate[e]) * value[e];
    free(gate); free(value);
    return 0;
}

/* ---- variants the paper's appendix defines on top of Eq. 3 ------------------------------------
 *
 * gate_fn   0: Swish (main paper)   1: GELU, z * Phi(z) with the exact Gaussian CDF   2: ReLU
 *           ("Other Activation Functions": g in Eq. 3 is replaced, nothing else changes)
 * mask_use  0: both branches masked (Eq. 3)
 *           1: dense gate   g(xW)        (.) x(Mbar (.) W)     ("Partial Mask Ablation", No Gate Mask)
 *           2: dense value  g(x(M (.) W)) (.) xW                (No Value Mask)
 *           3: no masks     g(xW)        (.) xW                 (No Masks)
 *           For n_m > 1 the per-mask terms are summed as in Eq. 3.
 * route     NULL, or double [T][n_m]: per-token weights G(x)_i multiplying route i
 *           ("Top-K Routing": MGLU_TopK(x) = sum_i G(x)_i g(x(M_i (.) W)) (.) x(Mbar_i (.) W)).
 */
static double gate_fn_apply(int gate_fn, double z)
{
    switch (gate_fn) {
    case 1: return 0.5 * z * (1.0 + erf(z / sqrt(2.0)));
    case 2: return z > 0.0 ? z : 0.0;
    default: return swish(z);
    }
}

int mglu_oracle_forward_variant(const double *x, const double *W, const uint8_t *M,
                                long T, long h, long d, long n_m, int gate_fn, int mask_use,
                                const double *route, double *out)
{
    if (!x || !W || !M || !out || T < 0 || h < 0 || d < 0 || n_m < 0) return 1;
    if (gate_fn < 0 || gate_fn > 2 || mask_use < 0 || mask_use > 3) return 1;
    const long hd = h * d, Td = T * d;
    for (long e = 0; e < Td; ++e) out[e] = 0.0;
    if (Td == 0 || n_m == 0) return 0;
    double *Wg = (double *)malloc(sizeof(double) * (size_t)(hd > 0 ? hd : 1));
    double *Wv = (double *)malloc(sizeof(double) * (size_t)(hd > 0 ? hd : 1));
    double *gate = (double *)malloc(sizeof(double) * (size_t)Td);
    double *value = (double *)malloc(sizeof(double) * (size_t)Td);
    if (!Wg || !Wv || !gate || !value) {
        free(Wg); free(Wv); free(gate); free(value);
        return 2;
    }
    const int dense_gate = (mask_use == 1 || mask_use == 3);
    const int dense_value = (mask_use == 2 || mask_use == 3);
    for (long i = 0; i < n_m; ++i) {
        const uint8_t *Mi = M + i * hd;
#pragma omp parallel for schedule(static)
        for (long e = 0; e < hd; ++e) {
            const double m = (double)(Mi[e] != 0);
            Wg[e] = dense_gate ? W[e] : m * W[e];
            Wv[e] = dense_value ? W[e] : (1.0 - m) * W[e];
        }
        matmul(x, Wg, gate, T, h, d);
        matmul(x, Wv, value, T, h, d);
        for (long tau = 0; tau < T; ++tau) {
            const double w = route ? route[tau * n_m + i] : 1.0;
            for (long j = 0; j < d; ++j)
                out[tau * d + j] += w * gate_fn_apply(gate_fn, gate[tau * d + j]) * value[tau * d + j];
        }
    }
    free(Wg); free(Wv); free(gate); free(value);
    return 0;
}

/* Router of the Top-K variant: logits l = x W_r (W_r double [h][n_m]); the K largest logits of each
 * token are kept (on equal logits the lower mask index wins), a softmax over the kept ones gives
 * the weights, every other weight is 0.  weights double [T][n_m]. */
int mglu_oracle_route_topk(const double *x, const double *Wr, long T, long h, long n_m, long K, double *weights)
{
    if (!x || !Wr || !weights || T < 0 || h < 0 || n_m < 1 || K < 1 || K > n_m) return 1;
    double *logit = (double *)malloc(sizeof(double) * (size_t)n_m);
    char *kept = (char *)malloc((size_t)n_m);
    if (!logit || !kept) { free(logit); free(kept); return 2; }
    for (long tau = 0; tau < T; ++tau) {
        for (long i = 0; i < n_m; ++i) {
            double acc = 0.0;
            for (long k = 0; k < h; ++k) acc += x[tau * h + k] * Wr[k * n_m + i];
            logit[i] = acc;
            kept[i] = 0;
        }
        for (long c = 0; c < K; ++c) {           /* pick the largest not yet kept, K times */
            long best = -1;
            for (long i = 0; i < n_m; ++i)
                if (!kept[i] && (best < 0 || logit[i] > logit[best])) best = i;
            kept[best] = 1;
        }
        double top = -INFINITY, sum = 0.0;
        for (long i = 0; i < n_m; ++i) if (kept[i] && logit[i] > top) top = logit[i];
        for (long i = 0; i < n_m; ++i) if (kept[i]) sum += exp(logit[i] - top);
        for (long i = 0; i < n_m; ++i) weights[tau * n_m + i] = kept[i] ? exp(logit[i] - top) / sum : 0.0;
    }
    free(logit); free(kept);
    return 0;
}

/* Output projection that follows the layer (Method, after Eq. 1: the intermediate representation is
 * mapped back by W_o in R^{d x h}): out[T][N] = a[T][K] W[K][N], a plain matrix product. */
int linear_oracle_forward(const double *a, const double *W, long T, long K, long N, double *out)
{
    if (!a || !W || !out || T < 0 || K < 0 || N < 0) return 1;
    matmul(a, W, out, T, K, N);
    return 0;
}

/* Number of threads the parallel loops above run on. */
int mglu_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
