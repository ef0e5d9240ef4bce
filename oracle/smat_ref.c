/* CPU oracle, plain C twin of the slow routines in smat_ref.py.
 *
 * TEST INFRASTRUCTURE, not product code: only tests/, __graft_entry__.smoke()
 * and the cpu_baseline leg of bench.py may load this file.  It shares no code
 * with the HIP library.  The loops below are the definitions written out; the
 * only parallelism is an OpenMP "for" over output rows in the product, which
 * does not change any row's summation order.
 *
 *   ref_spmm_f64          C = A.B and S = |A|.|B| in float64, CSR order
 *                         (Background section: C = AB, A sparse, B dense).
 *   ref_cluster_from_seed one round of the greedy Jaccard clustering
 *                         (Preprocessing section), literal scan over all rows.
 *   ref_jaccard_reorder   the rounds repeated until every row is clustered.
 *   ref_count_blocks      n_e of Eq. 2 for a given row order on the fixed
 *                         h-row grid (Blocked format section).
 *
 * The row "pattern" is the ascending set of block columns a row touches, given
 * as a CSR-like pair pat_ptr[M+1], pat_idx[].
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int ref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* C[i,j] = sum_p a[p] * b[col[p], j],  S[i,j] = sum_p |a[p]| * |b[col[p], j]|,
 * p running over the stored entries of row i in CSR order.  s may be NULL. */
void ref_spmm_f64(int64_t M, int64_t K, int64_t N,
                  const int64_t *row_ptr, const int32_t *col_idx, const double *a,
                  const double *b, double *c, double *s)
{
    (void)K;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < M; ++i) {
        double *ci = c + i * N;
        double *si = s ? s + i * N : NULL;
        for (int64_t j = 0; j < N; ++j) ci[j] = 0.0;
        if (si) for (int64_t j = 0; j < N; ++j) si[j] = 0.0;
        for (int64_t p = row_ptr[i]; p < row_ptr[i + 1]; ++p) {
            const double av = a[p];
            const double *bj = b + (int64_t)col_idx[p] * N;
            for (int64_t j = 0; j < N; ++j) ci[j] += av * bj[j];
            if (si) {
                const double aa = fabs(av);
                for (int64_t j = 0; j < N; ++j) si[j] += aa * fabs(bj[j]);
            }
        }
    }
}

/* One cluster.  in_pc[nbc] must be all zero on entry and is all zero on exit.
 * Merge test in integers:  1000*|w n pc| > (1000 - tau)*|w u pc|  <=>  J(w,pc) < tau/1000.
 * Two empty rows are at distance 0. */
int64_t ref_cluster_from_seed(int64_t M, const int64_t *pat_ptr, const int32_t *pat_idx,
                              int64_t nbc, int32_t tau_permille,
                              uint8_t *clustered, uint8_t *in_pc, int64_t v, int32_t *members)
{
    (void)nbc;
    int64_t n_members = 0, pc_size = 0;
    members[n_members++] = (int32_t)v;
    clustered[v] = 1;
    for (int64_t q = pat_ptr[v]; q < pat_ptr[v + 1]; ++q) { in_pc[pat_idx[q]] = 1; ++pc_size; }
    for (int64_t w = v + 1; w < M; ++w) {
        if (clustered[w]) continue;
        const int64_t wsize = pat_ptr[w + 1] - pat_ptr[w];
        int near;
        if (pc_size == 0 && wsize == 0) {
            near = tau_permille > 0;
        } else {
            int64_t inter = 0;
            for (int64_t q = pat_ptr[w]; q < pat_ptr[w + 1]; ++q) inter += in_pc[pat_idx[q]];
            const int64_t uni = wsize + pc_size - inter;
            near = 1000 * inter > (int64_t)(1000 - tau_permille) * uni;
        }
        if (near) {
            members[n_members++] = (int32_t)w;
            clustered[w] = 1;
            for (int64_t q = pat_ptr[w]; q < pat_ptr[w + 1]; ++q)
                if (!in_pc[pat_idx[q]]) { in_pc[pat_idx[q]] = 1; ++pc_size; }
        }
    }
    /* leave in_pc clean for the next cluster */
    for (int64_t m = 0; m < n_members; ++m) {
        const int64_t r = members[m];
        for (int64_t q = pat_ptr[r]; q < pat_ptr[r + 1]; ++q) in_pc[pat_idx[q]] = 0;
    }
    return n_members;
}

/* perm[new] = old; clusters in creation order, seeds in ascending row order.
 * Returns the number of clusters, or -1 on allocation failure / bad tau. */
int64_t ref_jaccard_reorder(int64_t M, const int64_t *pat_ptr, const int32_t *pat_idx,
                            int64_t nbc, int32_t tau_permille, int32_t *perm)
{
    if (tau_permille < 0 || tau_permille > 1000) return -1;
    uint8_t *clustered = (uint8_t *)calloc((size_t)(M > 0 ? M : 1), 1);
    uint8_t *in_pc = (uint8_t *)calloc((size_t)(nbc > 0 ? nbc : 1), 1);
    if (!clustered || !in_pc) { free(clustered); free(in_pc); return -1; }
    int64_t filled = 0, n_clusters = 0;
    for (int64_t v = 0; v < M; ++v) {
        if (clustered[v]) continue;
        filled += ref_cluster_from_seed(M, pat_ptr, pat_idx, nbc, tau_permille,
                                        clustered, in_pc, v, perm + filled);
        ++n_clusters;
    }
    free(clustered);
    free(in_pc);
    return n_clusters;
}

/* n_e for the row order perm on a grid of h-row block rows; -1 on allocation failure. */
int64_t ref_count_blocks(int64_t M, const int64_t *pat_ptr, const int32_t *pat_idx,
                         int64_t nbc, const int32_t *perm, int32_t h)
{
    int64_t *stamp = (int64_t *)malloc(sizeof(int64_t) * (size_t)(nbc > 0 ? nbc : 1));
    if (!stamp) return -1;
    for (int64_t j = 0; j < nbc; ++j) stamp[j] = -1;
    int64_t n_e = 0;
    for (int64_t i = 0; i < M; ++i) {
        const int64_t I = i / h, r = perm[i];
        for (int64_t q = pat_ptr[r]; q < pat_ptr[r + 1]; ++q)
            if (stamp[pat_idx[q]] != I) { stamp[pat_idx[q]] = I; ++n_e; }
    }
    free(stamp);
    return n_e;
}
