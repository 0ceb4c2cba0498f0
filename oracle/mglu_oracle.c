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

/* Number of threads the parallel loops above run on. */
int mglu_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
