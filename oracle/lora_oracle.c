/*
 * CPU checker for one multi-adapter LoRA projection.  TEST INFRASTRUCTURE ONLY:
 * nothing in the product path may call or link this file; it shares no code,
 * header, table or helper with the GPU library.
 *
 * What it computes (paper Sec. 2.2: a LoRA adapter adds two low-rank matrices to a
 * targeted layer and the adapter's activations are added to the backbone layer's
 * output; Sec. 1: adapters stay unmerged over one shared backbone; Sec. 2.2: several
 * adapters run inside one batch).  For token t with adapter i = id[t]:
 *
 *     y[t,n] = sum_k x[t,k] W[n,k]  +  s_i * sum_j ( sum_k x[t,k] A_i[j,k] ) B_i[n,j]
 *
 * and y[t,n] = sum_k x[t,k] W[n,k] when id[t] < 0 or rank_i == 0.  Where the backbone layer has a
 * bias b (the q, k, v projections of the Qwen2.5 family, one of the two model families of the
 * paper's evaluation, Sec. 8.1), the backbone layer's output is x W^T + b and the adapter's
 * activations are added to that: b[n] is added to every y[t,n], with or without an adapter.
 *
 * Inputs are bf16 bit patterns (uint16), widened exactly to double; all arithmetic is
 * IEEE double, plain nested loops in index order, no blocking, no intermediate or final
 * rounding.  Tokens are indexed directly by their adapter id: no grouping of tokens is
 * done here.
 *
 * Pins (tests, CPU only): all-backbone batches against a float64 library matmul, the
 * merged-weight identity y = x (W + s B A)^T, bitwise base-only results for B = 0 /
 * rank 0 / s = 0 / id = -1, hand-computed small-integer cases, one-hot inputs; for the bias:
 * x = 0 returns b in every row, a hand-computed integer case, and the difference to the
 * bias-free result on mixed batches.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double widen_bf16(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* Full output, y is [T, d_out] row-major double.  Adapter tables are indexed by adapter id
 * (0 .. n_adapters-1); A[i] is [rank[i], d_in], B[i] is [d_out, rank[i]], both row-major.
 * Returns 0, or -1 when a token names an id >= n_adapters or an adapter with missing data. */
int lora_oracle_project(int32_t T, int32_t d_in, int32_t d_out,
                        const uint16_t *x, const uint16_t *W, const int32_t *ids,
                        int32_t n_adapters, const int32_t *rank, const double *scale,
                        const uint16_t *const *A, const uint16_t *const *B,
                        const uint16_t *bias /* [d_out] or NULL */, double *y)
{
    for (int32_t t = 0; t < T; ++t) {
        int32_t i = ids[t];
        if (i >= n_adapters) return -1;
        if (i >= 0 && rank[i] > 0 && (A[i] == NULL || B[i] == NULL)) return -1;
    }
    int32_t rmax = 0;
    for (int32_t i = 0; i < n_adapters; ++i)
        if (rank[i] > rmax) rmax = rank[i];

#pragma omp parallel
    {
        double *v = (double *)malloc(sizeof(double) * (size_t)(rmax > 0 ? rmax : 1));
#pragma omp for schedule(dynamic, 1)
        for (int32_t t = 0; t < T; ++t) {
            const uint16_t *xt = x + (size_t)t * d_in;
            int32_t i = ids[t];
            int32_t r = (i >= 0) ? rank[i] : 0;
            for (int32_t j = 0; j < r; ++j) {
                const uint16_t *Aj = A[i] + (size_t)j * d_in;
                double acc = 0.0;
                for (int32_t k = 0; k < d_in; ++k)
                    acc += widen_bf16(xt[k]) * widen_bf16(Aj[k]);
                v[j] = acc;
            }
            for (int32_t n = 0; n < d_out; ++n) {
                const uint16_t *Wn = W + (size_t)n * d_in;
                double base = 0.0;
                for (int32_t k = 0; k < d_in; ++k)
                    base += widen_bf16(xt[k]) * widen_bf16(Wn[k]);
                if (bias) base += widen_bf16(bias[n]);
                if (r > 0) {
                    const uint16_t *Bn = B[i] + (size_t)n * r;
                    double d = 0.0;
                    for (int32_t j = 0; j < r; ++j)
                        d += v[j] * widen_bf16(Bn[j]);
                    y[(size_t)t * d_out + n] = base + scale[i] * d;
                } else {
                    y[(size_t)t * d_out + n] = base;
                }
            }
        }
        free(v);
    }
    return 0;
}

/* The same definition evaluated one output element at a time: y[q] for (ts[q], ns[q]). */
int lora_oracle_project_at(int32_t T, int32_t d_in, int32_t d_out,
                           const uint16_t *x, const uint16_t *W, const int32_t *ids,
                           int32_t n_adapters, const int32_t *rank, const double *scale,
                           const uint16_t *const *A, const uint16_t *const *B,
                           const uint16_t *bias /* [d_out] or NULL */, int64_t n_samples, const int32_t *ts, const int32_t *ns, double *y)
{
    for (int64_t q = 0; q < n_samples; ++q) {
        if (ts[q] < 0 || ts[q] >= T || ns[q] < 0 || ns[q] >= d_out) return -2;
        int32_t i = ids[ts[q]];
        if (i >= n_adapters) return -1;
        if (i >= 0 && rank[i] > 0 && (A[i] == NULL || B[i] == NULL)) return -1;
    }
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t q = 0; q < n_samples; ++q) {
        int32_t t = ts[q], n = ns[q];
        const uint16_t *xt = x + (size_t)t * d_in;
        const uint16_t *Wn = W + (size_t)n * d_in;
        int32_t i = ids[t];
        int32_t r = (i >= 0) ? rank[i] : 0;
        double base = 0.0;
        for (int32_t k = 0; k < d_in; ++k)
            base += widen_bf16(xt[k]) * widen_bf16(Wn[k]);
        if (bias) base += widen_bf16(bias[n]);
        if (r > 0) {
            const uint16_t *Bn = B[i] + (size_t)n * r;
            double d = 0.0;
            for (int32_t j = 0; j < r; ++j) {
                const uint16_t *Aj = A[i] + (size_t)j * d_in;
                double vj = 0.0;
                for (int32_t k = 0; k < d_in; ++k)
                    vj += widen_bf16(xt[k]) * widen_bf16(Aj[k]);
                d += vj * widen_bf16(Bn[j]);
            }
            y[q] = base + scale[i] * d;
        } else {
            y[q] = base;
        }
    }
    return 0;
}

int lora_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
