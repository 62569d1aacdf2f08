/*
 * Runs the CPU checker (oracle/lora_oracle.c, compiled into this executable with
 * -fsanitize=address,undefined) on one case read from a file, and writes what it returned.  TEST
 * INFRASTRUCTURE ONLY, like the checker itself.  Every array is copied into a heap block of exactly its own
 * size, so that an access one element outside it is an error the sanitizer reports.
 *
 * Case file (native endian):
 *   int32  T, d_in, d_out, n_adapters, has_bias, n_samples
 *   uint16 x[T*d_in], W[d_out*d_in];  int32 ids[T];  int32 rank[n_adapters];  double scale[n_adapters]
 *   per adapter with rank > 0:  uint16 A[rank*d_in], B[d_out*rank]
 *   uint16 bias[d_out] when has_bias;  int32 ts[n_samples], ns[n_samples]
 * Result file: int32 rc_full, rc_at;  double y[T*d_out];  double y_at[n_samples]
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int lora_oracle_project(int32_t T, int32_t d_in, int32_t d_out, const uint16_t *x, const uint16_t *W,
                        const int32_t *ids, int32_t n_adapters, const int32_t *rank, const double *scale,
                        const uint16_t *const *A, const uint16_t *const *B, const uint16_t *bias, double *y);
int lora_oracle_project_at(int32_t T, int32_t d_in, int32_t d_out, const uint16_t *x, const uint16_t *W,
                           const int32_t *ids, int32_t n_adapters, const int32_t *rank, const double *scale,
                           const uint16_t *const *A, const uint16_t *const *B, const uint16_t *bias,
                           int64_t n_samples, const int32_t *ts, const int32_t *ns, double *y);

static void *take(FILE *f, size_t count, size_t size)
{
    /* a block of exactly count*size bytes (one byte when that is zero, never touched) */
    void *p = malloc(count * size ? count * size : 1);
    if (!p || fread(p, size, count, f) != count) {
        fprintf(stderr, "oracle_driver: short case file\n");
        exit(3);
    }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: oracle_driver <case file> <result file>\n");
        return 2;
    }
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int32_t *h = take(f, 6, sizeof(int32_t));
    const int32_t T = h[0], d_in = h[1], d_out = h[2], n_ad = h[3], has_bias = h[4], n_samples = h[5];
    uint16_t *x = take(f, (size_t)T * d_in, 2);
    uint16_t *W = take(f, (size_t)d_out * d_in, 2);
    int32_t *ids = take(f, T, 4);
    int32_t *rank = take(f, n_ad, 4);
    double *scale = take(f, n_ad, 8);
    const uint16_t **A = calloc(n_ad ? n_ad : 1, sizeof *A);
    const uint16_t **B = calloc(n_ad ? n_ad : 1, sizeof *B);
    for (int32_t i = 0; i < n_ad; ++i)
        if (rank[i] > 0) {
            A[i] = take(f, (size_t)rank[i] * d_in, 2);
            B[i] = take(f, (size_t)d_out * rank[i], 2);
        }
    uint16_t *bias = has_bias ? take(f, d_out, 2) : NULL;
    int32_t *ts = take(f, n_samples, 4);
    int32_t *ns = take(f, n_samples, 4);
    fclose(f);

    double *y = malloc((size_t)T * d_out * 8 ? (size_t)T * d_out * 8 : 1);
    double *y_at = malloc(n_samples ? (size_t)n_samples * 8 : 1);
    int32_t rc[2];
    rc[0] = lora_oracle_project(T, d_in, d_out, x, W, ids, n_ad, rank, scale, A, B, bias, y);
    rc[1] = lora_oracle_project_at(T, d_in, d_out, x, W, ids, n_ad, rank, scale, A, B, bias, n_samples, ts, ns, y_at);

    FILE *o = fopen(argv[2], "wb");
    if (!o) return 2;
    fwrite(rc, 4, 2, o);
    if (rc[0] == 0) fwrite(y, 8, (size_t)T * d_out, o);
    if (rc[1] == 0) fwrite(y_at, 8, n_samples, o);
    fclose(o);

    for (int32_t i = 0; i < n_ad; ++i) {
        free((void *)A[i]);
        free((void *)B[i]);
    }
    free(A); free(B); free(h); free(x); free(W); free(ids); free(rank); free(scale); free(bias); free(ts); free(ns);
    free(y); free(y_at);
    return 0;
}
