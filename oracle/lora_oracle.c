/*
 * CPU oracle for the multi-LoRA batched linear layer.  TEST INFRASTRUCTURE ONLY:
 * nothing on the product path may call, link or import this file; it shares no
 * code with the HIP kernels.
 *
 * What it computes (paper section 2.2 and section 4.4, "unmerged" LoRA
 * inference: the backbone product and the adapter product are computed
 * separately on a read-only backbone and then summed; section 5 repeats it
 * for the implementation).  Written out for a batch in which every request
 * carries its own adapter, for every token row t of request i(t) with adapter
 * a = req_adapter[i(t)]:
 *
 *     Y[t,n] = sum_k X[t,k] W0[k,n]
 *            + s_a * sum_j ( sum_k X[t,k] A_a[k,j] ) B_a[j,n]        (a >= 0)
 *     Y[t,n] = sum_k X[t,k] W0[k,n]                                   (a == -1)
 *
 * Everything is IEEE fp64.  Inputs are the stored bit patterns (fp32, or bf16
 * as uint16) widened exactly.  Sums run in ascending index order (k, then j),
 * products are rounded before they are added (built with -ffp-contract=off),
 * and each row is computed independently of every other row.  There is no
 * blocking, no segment building and no reordering: requests are walked in the
 * order given.
 *
 * Storage (as PyTorch / PEFT hold the tensors):
 *     X  [T, ldx]   row t at X + t*ldx, K used
 *     W0 [N, ldw]   W0[k,n] of the formula is stored at W0[n*ldw + k]
 *     A_a[r_a, K]   A_a[k,j] is stored at A_a[j*K + k]
 *     B_a[N, r_a]   B_a[j,n] is stored at B_a[n*r_a + j]
 *
 * Parity pins (tests/test_oracle_pins.py): zero-B equals the base product bit
 * for bit; a one-adapter batch equals X (W0 + s A B) with the merged matrix
 * formed in fp64; request permutation and batch-of-one invariance, bit for
 * bit; exact integer brute force on tiny shapes; linearity in s and in X; a
 * rank-one closed form; the closed-form output RMS of the benchmark
 * distributions; a library fp64 matmul of the same three products.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

static inline double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == ORACLE_BF16) {
        uint32_t u = ((uint32_t)((const uint16_t *)base)[idx]) << 16;
        float f;
        memcpy(&f, &u, sizeof f);
        return (double)f;
    }
    return (double)((const float *)base)[idx];
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * rows == NULL: compute all T rows, output row t at Y + t*ldy.
 * rows != NULL: compute only rows[0..n_rows), output i at Y + i*ldy.
 * V (optional, may be NULL): the *unscaled* intermediate sum_k X[t,k] A_a[k,j],
 * written at V + i*ldv + j for j < r_a (entries j >= r_a are set to 0).
 * Returns 0, or a negative code: -1 bad adapter id, -2 negative length,
 * -3 sum of lengths != T, -4 row index out of range, -5 adapter used but
 * rank <= 0 or null weights, -6 bad dtype / null argument.
 */
int oracle_lora_linear(int dtype, int64_t T, int32_t K, int32_t N,
                       const void *X, int64_t ldx,
                       const void *W0, int64_t ldw,
                       int32_t n_req, const int32_t *req_adapter, const int32_t *req_ntok,
                       int32_t n_adapters, const void *const *A, const void *const *B,
                       const int32_t *rank, const float *scale,
                       const int64_t *rows, int64_t n_rows,
                       double *Y, int64_t ldy,
                       double *V, int64_t ldv)
{
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16)
        return -6;
    if (T < 0 || K < 0 || N < 0 || n_req < 0 || (n_req > 0 && (!req_adapter || !req_ntok)))
        return -6;

    /* adapter of every token row, walking the requests in submission order */
    int32_t *row_ad = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1));
    if (!row_ad)
        return -6;
    int64_t t = 0;
    for (int32_t i = 0; i < n_req; ++i) {
        int32_t a = req_adapter[i], L = req_ntok[i];
        if (a < -1 || a >= n_adapters) { free(row_ad); return -1; }
        if (L < 0) { free(row_ad); return -2; }
        if (t + L > T) { free(row_ad); return -3; }
        if (L > 0 && a >= 0 && (rank[a] <= 0 || !A[a] || !B[a])) { free(row_ad); return -5; }
        for (int32_t q = 0; q < L; ++q)
            row_ad[t++] = a;
    }
    if (t != T) { free(row_ad); return -3; }

    const int64_t n_out = rows ? n_rows : T;
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t r = rows ? rows[i] : i;
        if (r < 0 || r >= T) { free(row_ad); return -4; }
    }
    if (n_out > 0 && (!X || !W0 || !Y)) { free(row_ad); return -6; }

    int32_t r_cap = 1;
    for (int32_t a = 0; a < n_adapters; ++a)
        if (rank[a] > r_cap)
            r_cap = rank[a];

#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * (size_t)(K > 0 ? K : 1));
        double *v = (double *)malloc(sizeof(double) * (size_t)r_cap);
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < n_out; ++i) {
            const int64_t row = rows ? rows[i] : i;
            const int32_t a = row_ad[row];
            for (int32_t k = 0; k < K; ++k)
                x[k] = load_elem(X, row * ldx + k, dtype);

            int32_t r = 0;
            double s = 0.0;
            if (a >= 0) {
                r = rank[a];
                s = (double)scale[a];
                /* shrink: v_j = sum_k x_k A_a[k,j] */
                for (int32_t j = 0; j < r; ++j) {
                    double acc = 0.0;
                    for (int32_t k = 0; k < K; ++k)
                        acc += x[k] * load_elem(A[a], (int64_t)j * K + k, dtype);
                    v[j] = acc;
                }
            }
            if (V) {
                for (int64_t j = 0; j < ldv; ++j)
                    V[i * ldv + j] = (j < r) ? v[j] : 0.0;
            }
            for (int32_t n = 0; n < N; ++n) {
                /* backbone product */
                double base = 0.0;
                for (int32_t k = 0; k < K; ++k)
                    base += x[k] * load_elem(W0, (int64_t)n * ldw + k, dtype);
                if (a >= 0) {
                    /* adapter product, scaled after the rank-r contraction */
                    double lo = 0.0;
                    for (int32_t j = 0; j < r; ++j)
                        lo += v[j] * load_elem(B[a], (int64_t)n * r + j, dtype);
                    Y[i * ldy + n] = base + s * lo;
                } else {
                    Y[i * ldy + n] = base;
                }
            }
        }
        free(x);
        free(v);
    }
    free(row_ad);
    return 0;
}
