/*
 * CPU oracle for sparse-times-dense tensor contractions.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct definition that the GPU library is
 * checked against.  It shares no code, header, table or helper with the HIP
 * path and must never be linked into, imported by or called from the product
 * library; only the tests, the smoke check and the benchmark's CPU-baseline
 * leg may use it.
 *
 * Every function evaluates the plain (perfectly nested, "linear") loop nest of
 * the contraction -- one iteration per stored nonzero per dense index -- in
 * fp64.  All fused / fissioned schedules of a contraction are members of one
 * equivalence class and must produce exactly this result up to rounding
 * (Section 4.1, "equivalence class"; Section 4.5, "Equivalence of BIG and
 * LIG"), so the linear nest is the definition of what every schedule computes.
 *
 * The sparse operand is given as COO (one int32 coordinate array per mode and
 * one value array), in ANY order; duplicates are summed.  The nonzeros are
 * bucketed by their first coordinate with a stable counting sort so that the
 * outermost loop can run over output rows i; rows are disjoint in the output,
 * so the OpenMP loop over i needs no atomics and the summation order inside a
 * row is the storage order of the input.  There is no blocking, fusion or
 * reordering beyond that.
 *
 * Dense operands are row-major with the rank index contiguous, as in the
 * generated code of Figure 1b (C_vals[j * C2_dimension + k]).
 *
 * Pins (tests/test_oracle_pins.py): brute-force dense einsum on tiny tensors,
 * a hand-computed worked example (tests/golden), linearity in each factor,
 * closed forms (all-ones / one-hot / identity factors), reduction to SpMM and
 * to (X Y^T) Z, and invariance under permutation of the COO order.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Stable counting sort of nonzero positions by first coordinate.
 * row_ptr has I+1 entries, perm has nnz entries.  Returns 0 on success. */
static int bucket_by_row(int64_t nnz, const int32_t *ci, int64_t I, int64_t **row_ptr_out, int64_t **perm_out)
{
    int64_t *row_ptr = (int64_t *)calloc((size_t)I + 2, sizeof(int64_t));
    int64_t *perm = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nnz > 0 ? nnz : 1));
    if (!row_ptr || !perm) { free(row_ptr); free(perm); return -1; }
    for (int64_t n = 0; n < nnz; ++n) {
        if (ci[n] < 0 || ci[n] >= I) { free(row_ptr); free(perm); return -2; }
        row_ptr[ci[n] + 2]++;
    }
    for (int64_t i = 0; i < I; ++i) row_ptr[i + 2] += row_ptr[i + 1];
    /* row_ptr[i+1] is now the running insert cursor of row i */
    for (int64_t n = 0; n < nnz; ++n) perm[row_ptr[ci[n] + 1]++] = n;
    /* after the fill, row_ptr[i+1] == end of row i == start of row i+1; row_ptr[0]==0 */
    *row_ptr_out = row_ptr;
    *perm_out = perm;
    return 0;
}

/*
 * Table 2, kernel 6 <SpTTM,TTM>:  A(i,l,m) = sum_{j,k} B(i,j,k) * C(j,l) * D(k,m).
 * A is I x L x M (fully overwritten), C is J x L, D is K x M.
 */
int oracle_ttmc3(int64_t nnz, const int32_t *ci, const int32_t *cj, const int32_t *ck, const double *vals,
                 int64_t I, int64_t J, int64_t K, const double *C, int64_t L, const double *D, int64_t M,
                 double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J || ck[n] < 0 || ck[n] >= K) { free(row_ptr); free(perm); return -2; }
    memset(A, 0, sizeof(double) * (size_t)(I * L * M));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * L * M;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t n = perm[q];
            const double b = vals[n];
            const double *Cj = C + (int64_t)cj[n] * L;
            const double *Dk = D + (int64_t)ck[n] * M;
            for (int64_t l = 0; l < L; ++l)
                for (int64_t m = 0; m < M; ++m)
                    Ai[l * M + m] += b * Cj[l] * Dk[m];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}

/*
 * MTTKRP (the producer of Table 2, kernel 8; described in Section 6):
 * A(i,r) = sum_{j,k} B(i,j,k) * C(j,r) * D(k,r).   A is I x R, C is J x R, D is K x R.
 */
int oracle_mttkrp3(int64_t nnz, const int32_t *ci, const int32_t *cj, const int32_t *ck, const double *vals,
                   int64_t I, int64_t J, int64_t K, const double *C, const double *D, int64_t R,
                   double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J || ck[n] < 0 || ck[n] >= K) { free(row_ptr); free(perm); return -2; }
    memset(A, 0, sizeof(double) * (size_t)(I * R));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * R;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t n = perm[q];
            const double b = vals[n];
            const double *Cj = C + (int64_t)cj[n] * R;
            const double *Dk = D + (int64_t)ck[n] * R;
            for (int64_t r = 0; r < R; ++r)
                Ai[r] += b * Cj[r] * Dk[r];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}

/*
 * Table 2, kernel 1 <SDDMM,SpMM>:
 * A(i,l) = sum_j S(i,j) * ( sum_k X(i,k) * Y(j,k) ) * Z(j,l).
 * S is I x J sparse, X is I x K, Y is J x K, Z is J x L, A is I x L.
 * The inner sum over k is evaluated first for each stored (i,j), as the
 * expression is parenthesised.
 */
int oracle_sddmm_spmm(int64_t nnz, const int32_t *ci, const int32_t *cj, const double *vals,
                      int64_t I, int64_t J, const double *X, const double *Y, int64_t K,
                      const double *Z, int64_t L, double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J) { free(row_ptr); free(perm); return -2; }
    memset(A, 0, sizeof(double) * (size_t)(I * L));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * L;
        const double *Xi = X + i * K;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t n = perm[q];
            const double *Yj = Y + (int64_t)cj[n] * K;
            const double *Zj = Z + (int64_t)cj[n] * L;
            double dot = 0.0;
            for (int64_t k = 0; k < K; ++k) dot += Xi[k] * Yj[k];
            const double t = vals[n] * dot;
            for (int64_t l = 0; l < L; ++l) Ai[l] += t * Zj[l];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}

/*
 * Order-4 TTM chain (the recursion of Section 4.2 applied twice to an order-4 operand):
 * A(i,l,m,n) = sum_{j,k,p} B(i,j,k,p) * C(j,l) * D(k,m) * E(p,n).
 * A is I x L x M x N, C is J x L, D is K x M, E is P x N.
 */
int oracle_ttmc4(int64_t nnz, const int32_t *ci, const int32_t *cj, const int32_t *ck, const int32_t *cp,
                 const double *vals, int64_t I, int64_t J, int64_t K, int64_t P,
                 const double *C, int64_t L, const double *D, int64_t M, const double *E, int64_t N,
                 double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J || ck[n] < 0 || ck[n] >= K || cp[n] < 0 || cp[n] >= P) {
            free(row_ptr); free(perm); return -2;
        }
    memset(A, 0, sizeof(double) * (size_t)(I * L * M * N));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * L * M * N;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t z = perm[q];
            const double b = vals[z];
            const double *Cj = C + (int64_t)cj[z] * L;
            const double *Dk = D + (int64_t)ck[z] * M;
            const double *Ep = E + (int64_t)cp[z] * N;
            for (int64_t l = 0; l < L; ++l)
                for (int64_t m = 0; m < M; ++m)
                    for (int64_t n = 0; n < N; ++n)
                        Ai[(l * M + m) * N + n] += b * Cj[l] * Dk[m] * Ep[n];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}

/*
 * Table 2, kernel 5 <3D TTMC> (the running example of Sections 1 and 3, Figure 2a):
 * A(l,m,n) = sum_{i,j,k} B(i,j,k) * C(i,l) * D(j,m) * E(k,n).
 * A is L x M x N, C is I x L, D is J x M, E is K x N.  The output carries no sparse index, so
 * the outermost loop here is the dense index l (the perfectly nested loop of Figure 2a may
 * take its six loops in any order that respects the sparse operand's level order): threads
 * own disjoint slabs A(l,:,:) and every slab sums the stored entries in storage order.
 */
int oracle_ttmc_all(int64_t nnz, const int32_t *ci, const int32_t *cj, const int32_t *ck, const double *vals,
                    int64_t I, int64_t J, int64_t K, const double *C, int64_t L, const double *D, int64_t M,
                    const double *E, int64_t N, double *A, int nthreads)
{
    for (int64_t z = 0; z < nnz; ++z)
        if (ci[z] < 0 || ci[z] >= I || cj[z] < 0 || cj[z] >= J || ck[z] < 0 || ck[z] >= K) return -2;
    memset(A, 0, sizeof(double) * (size_t)(L * M * N));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(static) num_threads(nthreads)
    for (int64_t l = 0; l < L; ++l) {
        double *Al = A + l * M * N;
        for (int64_t z = 0; z < nnz; ++z) {
            const double b = vals[z];
            const double c = C[(int64_t)ci[z] * L + l];
            const double *Dj = D + (int64_t)cj[z] * M;
            const double *Ek = E + (int64_t)ck[z] * N;
            for (int64_t m = 0; m < M; ++m)
                for (int64_t n = 0; n < N; ++n)
                    Al[m * N + n] += b * c * Dj[m] * Ek[n];
        }
    }
    return 0;
}

/*
 * Table 2, kernel 8 <MTTKRP,GEMM>:
 * A(i,m) = sum_{j,k,r} B(i,j,k) * C(j,r) * D(k,r) * E(r,m).
 * A is I x M, C is J x R, D is K x R, E is R x M.
 */
int oracle_mttkrp_gemm(int64_t nnz, const int32_t *ci, const int32_t *cj, const int32_t *ck, const double *vals,
                       int64_t I, int64_t J, int64_t K, const double *C, const double *D, int64_t R,
                       const double *E, int64_t M, double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J || ck[n] < 0 || ck[n] >= K) { free(row_ptr); free(perm); return -2; }
    memset(A, 0, sizeof(double) * (size_t)(I * M));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * M;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t n = perm[q];
            const double b = vals[n];
            const double *Cj = C + (int64_t)cj[n] * R;
            const double *Dk = D + (int64_t)ck[n] * R;
            for (int64_t r = 0; r < R; ++r)
                for (int64_t m = 0; m < M; ++m)
                    Ai[m] += b * Cj[r] * Dk[r] * E[r * M + m];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}

/*
 * Table 2, kernel 2 <SDDMM,SpMM,GEMM>:
 * A(i,m) = sum_{j,k,l} S(i,j) * X(i,k) * Y(j,k) * Z(j,l) * F(l,m).
 * S is I x J sparse, X is I x K, Y is J x K, Z is J x L, F is L x M, A is I x M.
 * The perfectly nested loop: every stored entry times one element of every factor for every
 * combination of k, l and m.
 */
int oracle_sddmm_spmm_gemm(int64_t nnz, const int32_t *ci, const int32_t *cj, const double *vals,
                           int64_t I, int64_t J, const double *X, const double *Y, int64_t K,
                           const double *Z, int64_t L, const double *F, int64_t M, double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J) { free(row_ptr); free(perm); return -2; }
    memset(A, 0, sizeof(double) * (size_t)(I * M));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * M;
        const double *Xi = X + i * K;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t n = perm[q];
            const double *Yj = Y + (int64_t)cj[n] * K;
            const double *Zj = Z + (int64_t)cj[n] * L;
            for (int64_t k = 0; k < K; ++k)
                for (int64_t l = 0; l < L; ++l)
                    for (int64_t m = 0; m < M; ++m)
                        Ai[m] += vals[n] * Xi[k] * Yj[k] * Zj[l] * F[l * M + m];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}

/*
 * SpMM, the loop of Figure 1b:  A(i,k) = sum_j B(i,j) * C(j,k).
 * Kept as the degenerate order-2 member of the family; used to pin the others.
 */
int oracle_spmm(int64_t nnz, const int32_t *ci, const int32_t *cj, const double *vals,
                int64_t I, int64_t J, const double *C, int64_t K, double *A, int nthreads)
{
    int64_t *row_ptr, *perm;
    int rc = bucket_by_row(nnz, ci, I, &row_ptr, &perm);
    if (rc) return rc;
    for (int64_t n = 0; n < nnz; ++n)
        if (cj[n] < 0 || cj[n] >= J) { free(row_ptr); free(perm); return -2; }
    memset(A, 0, sizeof(double) * (size_t)(I * K));
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
    for (int64_t i = 0; i < I; ++i) {
        double *Ai = A + i * K;
        for (int64_t q = row_ptr[i]; q < row_ptr[i + 1]; ++q) {
            const int64_t n = perm[q];
            const double *Cj = C + (int64_t)cj[n] * K;
            for (int64_t k = 0; k < K; ++k) Ai[k] += vals[n] * Cj[k];
        }
    }
    free(row_ptr); free(perm);
    return 0;
}
