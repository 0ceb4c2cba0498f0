/*
 * Test infrastructure: runs every entry point of the CPU oracle under AddressSanitizer and
 * UndefinedBehaviorSanitizer (tests/test_oracle_sanitizers.py compiles this file with
 * -fsanitize=address,undefined and compares what it writes with the regular oracle build).
 * It holds no arithmetic of its own: it reads the inputs from a file, calls the oracle
 * (compiled into this program from its one source file), and writes the results back.
 *
 * Input file:  6 int64 (T, h, d, n_m, K, has_route), then doubles x[T*h], W[h*d], W2[h*d],
 *              Wr[h*n_m], route[T*n_m], then n_m*h*d mask bytes.
 * Output file: doubles out[T*d], gate[n_m*T*d], value[n_m*T*d], swiglu[T*d], variant[T*d]
 *              (GELU gate, dense value, routed if has_route), weights[T*n_m], linear[T*d].
 */
#include <stdio.h>

#include "../oracle/mglu_oracle.c"

static void *must(void *p) { if (!p) { fprintf(stderr, "out of memory\n"); exit(3); } return p; }

int main(int argc, char **argv)
{
    if (argc != 3) { fprintf(stderr, "usage: %s in out\n", argv[0]); return 2; }
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int64_t hdr[6];
    if (fread(hdr, sizeof(int64_t), 6, f) != 6) return 2;
    const long T = hdr[0], h = hdr[1], d = hdr[2], n_m = hdr[3], K = hdr[4], has_route = hdr[5];
    double *x = must(malloc(sizeof(double) * (size_t)(T * h + 1)));
    double *W = must(malloc(sizeof(double) * (size_t)(h * d + 1)));
    double *W2 = must(malloc(sizeof(double) * (size_t)(h * d + 1)));
    double *Wr = must(malloc(sizeof(double) * (size_t)(h * n_m + 1)));
    double *route = must(malloc(sizeof(double) * (size_t)(T * n_m + 1)));
    uint8_t *M = must(malloc((size_t)(n_m * h * d + 1)));
    if (fread(x, sizeof(double), (size_t)(T * h), f) != (size_t)(T * h)) return 2;
    if (fread(W, sizeof(double), (size_t)(h * d), f) != (size_t)(h * d)) return 2;
    if (fread(W2, sizeof(double), (size_t)(h * d), f) != (size_t)(h * d)) return 2;
    if (fread(Wr, sizeof(double), (size_t)(h * n_m), f) != (size_t)(h * n_m)) return 2;
    if (fread(route, sizeof(double), (size_t)(T * n_m), f) != (size_t)(T * n_m)) return 2;
    if (fread(M, 1, (size_t)(n_m * h * d), f) != (size_t)(n_m * h * d)) return 2;
    fclose(f);

    const size_t Td = (size_t)(T * d);
    double *out = must(malloc(sizeof(double) * (Td + 1)));
    double *gate = must(malloc(sizeof(double) * ((size_t)n_m * Td + 1)));
    double *value = must(malloc(sizeof(double) * ((size_t)n_m * Td + 1)));
    double *sw = must(malloc(sizeof(double) * (Td + 1)));
    double *var = must(malloc(sizeof(double) * (Td + 1)));
    double *wts = must(malloc(sizeof(double) * ((size_t)(T * n_m) + 1)));
    double *lin = must(malloc(sizeof(double) * (Td + 1)));
    int rc = 0;
    rc |= mglu_oracle_forward(x, W, M, T, h, d, n_m, out, gate, value);
    rc |= swiglu_oracle_forward(x, W, W2, T, h, d, sw);
    rc |= mglu_oracle_forward_variant(x, W, M, T, h, d, n_m, 1, 2, has_route ? route : NULL, var);
    rc |= mglu_oracle_route_topk(x, Wr, T, h, n_m, K, wts);
    rc |= linear_oracle_forward(x, W, T, h, d, lin);
    if (rc) { fprintf(stderr, "an oracle call failed\n"); return 4; }

    f = fopen(argv[2], "wb");
    if (!f) return 2;
    fwrite(out, sizeof(double), Td, f);
    fwrite(gate, sizeof(double), (size_t)n_m * Td, f);
    fwrite(value, sizeof(double), (size_t)n_m * Td, f);
    fwrite(sw, sizeof(double), Td, f);
    fwrite(var, sizeof(double), Td, f);
    fwrite(wts, sizeof(double), (size_t)(T * n_m), f);
    fwrite(lin, sizeof(double), Td, f);
    fclose(f);
    free(x); free(W); free(W2); free(Wr); free(route); free(M);
    free(out); free(gate); free(value); free(sw); free(var); free(wts); free(lin);
    return 0;
}
