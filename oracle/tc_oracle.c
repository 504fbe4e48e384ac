/*
 * CPU oracle for fp64 tensor contraction -- TEST INFRASTRUCTURE, not the product.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may use this
 * file.  It shares no code with the HIP library and is deliberately plain:
 * fp64 throughout, no Strassen, no reordering beyond what is stated below.
 *
 *   orc_contract_literal  the definition of tensor contraction (paper, Sec. 2.3
 *                         "Tensor Contraction", the displayed definition with
 *                         alpha and beta) with element locations from the general
 *                         stride layout (Sec. 2.3 "General stride layouts").
 *   orc_scatter           scatter vector of an index bundle (Sec. 2.3 "Block Scatter
 *                         Matrix View", the rscat formula).
 *   orc_block_scatter     block scatter vector: the common stride of each block of
 *                         blk consecutive scatter entries, 0 if irregular (same section).
 *   orc_contract_rows     the same sum as orc_contract_literal written on the matrix
 *                         view (LOC = rscat_i + cscat_j, the scatter-matrix location
 *                         formula of Sec. 2.3); rows may be a subset.  Cache-tiled and OpenMP-parallel; every C element is
 *                         still one thread's running sum over p = 0..k-1 in order.
 *   orc_matvec            y = M x on a matrix view (for the Freivalds check).
 *
 * Pins: tests/test_oracle_*.py (numpy einsum / matmul, brute force, the paper's
 * worked layout example, invariants).
 */
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_OK = 0, ORC_ERR_LABEL = -1, ORC_ERR_LENGTH = -2, ORC_ERR_NDIM = -3, ORC_ERR_ALLOC = -4 };

#define ORC_MAXD 32

/* threads the OpenMP loops below will use */
int orc_num_threads(void) { return omp_get_max_threads(); }

static int find_label(const char *idx, int nd, char c)
{
    for (int d = 0; d < nd; ++d)
        if (idx[d] == c)
            return d;
    return -1;
}

/* C[..] = alpha * sum_P A[..] * B[..] + beta * C[..]; beta == 0 does not read C. */
int orc_contract_literal(int ndA, const int64_t *lenA, const int64_t *strA, const char *idxA, const double *A,
                         int ndB, const int64_t *lenB, const int64_t *strB, const char *idxB, const double *B,
                         int ndC, const int64_t *lenC, const int64_t *strC, const char *idxC, double *C,
                         double alpha, double beta)
{
    if (ndA > ORC_MAXD || ndB > ORC_MAXD || ndC > ORC_MAXD || ndA < 0 || ndB < 0 || ndC < 0)
        return ORC_ERR_NDIM;
    /* every label occurs once per tensor and in exactly two tensors */
    for (int d = 0; d < ndA; ++d) {
        if (find_label(idxA, d, idxA[d]) >= 0)
            return ORC_ERR_LABEL;
        int b = find_label(idxB, ndB, idxA[d]), c = find_label(idxC, ndC, idxA[d]);
        if ((b >= 0) == (c >= 0))
            return ORC_ERR_LABEL;
        if (b >= 0 && lenB[b] != lenA[d])
            return ORC_ERR_LENGTH;
        if (c >= 0 && lenC[c] != lenA[d])
            return ORC_ERR_LENGTH;
    }
    for (int d = 0; d < ndB; ++d) {
        if (find_label(idxB, d, idxB[d]) >= 0)
            return ORC_ERR_LABEL;
        int a = find_label(idxA, ndA, idxB[d]), c = find_label(idxC, ndC, idxB[d]);
        if ((a >= 0) == (c >= 0))
            return ORC_ERR_LABEL;
        if (c >= 0 && lenC[c] != lenB[d])
            return ORC_ERR_LENGTH;
    }
    for (int d = 0; d < ndC; ++d) {
        if (find_label(idxC, d, idxC[d]) >= 0)
            return ORC_ERR_LABEL;
        int a = find_label(idxA, ndA, idxC[d]), b = find_label(idxB, ndB, idxC[d]);
        if ((a >= 0) == (b >= 0))
            return ORC_ERR_LABEL;
    }
    /* contracted labels, in A's order */
    int nP = 0, pA[ORC_MAXD], pB[ORC_MAXD];
    int64_t lenP[ORC_MAXD];
    for (int d = 0; d < ndA; ++d) {
        int b = find_label(idxB, ndB, idxA[d]);
        if (b >= 0) {
            pA[nP] = d;
            pB[nP] = b;
            lenP[nP] = lenA[d];
            ++nP;
        }
    }
    int64_t nC = 1, nPtot = 1;
    for (int d = 0; d < ndC; ++d)
        nC *= lenC[d];
    for (int q = 0; q < nP; ++q)
        nPtot *= lenP[q];
    if (nC == 0)
        return ORC_OK;

    int64_t val[256];
    memset(val, 0, sizeof val);
    int64_t ci[ORC_MAXD], pi[ORC_MAXD];
    memset(ci, 0, sizeof ci);
    for (int64_t e = 0; e < nC; ++e) {
        for (int d = 0; d < ndC; ++d)
            val[(unsigned char)idxC[d]] = ci[d];
        int64_t locC = 0;
        for (int d = 0; d < ndC; ++d)
            locC += ci[d] * strC[d];
        double sum = 0.0;
        memset(pi, 0, sizeof pi);
        for (int64_t p = 0; p < nPtot; ++p) {
            for (int q = 0; q < nP; ++q)
                val[(unsigned char)idxA[pA[q]]] = pi[q];
            int64_t locA = 0, locB = 0;
            for (int d = 0; d < ndA; ++d)
                locA += val[(unsigned char)idxA[d]] * strA[d];
            for (int d = 0; d < ndB; ++d)
                locB += val[(unsigned char)idxB[d]] * strB[d];
            sum += A[locA] * B[locB];
            for (int q = 0; q < nP; ++q) { /* odometer, first contracted label fastest */
                if (++pi[q] < lenP[q])
                    break;
                pi[q] = 0;
            }
        }
        (void)pB;
        C[locC] = (beta == 0.0) ? alpha * sum : alpha * sum + beta * C[locC];
        for (int d = 0; d < ndC; ++d) {
            if (++ci[d] < lenC[d])
                break;
            ci[d] = 0;
        }
    }
    return ORC_OK;
}

/* out[i] = sum_k i_k * stride_k with i = sum_k i_k * prod_{l<k} len_l (first index fastest). */
int orc_scatter(int nb, const int64_t *len, const int64_t *stride, int64_t *out)
{
    if (nb < 0 || nb > ORC_MAXD)
        return ORC_ERR_NDIM;
    int64_t total = 1;
    for (int d = 0; d < nb; ++d)
        total *= len[d];
    int64_t cur[ORC_MAXD];
    memset(cur, 0, sizeof cur);
    for (int64_t i = 0; i < total; ++i) {
        int64_t loc = 0;
        for (int d = 0; d < nb; ++d)
            loc += cur[d] * stride[d];
        out[i] = loc;
        for (int d = 0; d < nb; ++d) {
            if (++cur[d] < len[d])
                break;
            cur[d] = 0;
        }
    }
    return ORC_OK;
}

/* out[b] = s if scat[e+1]-scat[e] == s for all consecutive entries of block b, else 0.
 * A block holding a single entry has no stride to contradict; it is recorded as regular with stride 1. */
int orc_block_scatter(const int64_t *scat, int64_t n, int64_t blk, int64_t *out)
{
    if (blk <= 0)
        return ORC_ERR_LENGTH;
    for (int64_t b = 0; b * blk < n; ++b) {
        int64_t lo = b * blk, hi = lo + blk < n ? lo + blk : n;
        int64_t s = (hi - lo >= 2) ? scat[lo + 1] - scat[lo] : 1;
        for (int64_t e = lo + 1; e < hi; ++e)
            if (scat[e] - scat[e - 1] != s)
                s = 0;
        out[b] = s;
    }
    return ORC_OK;
}

#define MR 4
#define NR 8
#define KC 1024
#define NC 64
#define MCH 256

/* out[r*n + j] = alpha * sum_p A[rsA[rows[r]] + csA[p]] * B[rsB[p] + csB[j]] + beta * C0[rsC[rows[r]] + csC[j]]
 * rows == NULL means rows 0..nrows-1.  C0 is not read when beta == 0. */
int orc_contract_rows(const double *A, const double *B, const double *C0,
                      const int64_t *rsA, const int64_t *csA, const int64_t *rsB, const int64_t *csB,
                      const int64_t *rsC, const int64_t *csC,
                      const int64_t *rows, int64_t nrows, int64_t n, int64_t k, double alpha, double beta, double *out)
{
    if (nrows <= 0 || n <= 0)
        return ORC_OK;
    memset(out, 0, sizeof(double) * (size_t)nrows * (size_t)n);
    int64_t nct = (n + NC - 1) / NC, nrc = (nrows + MCH - 1) / MCH;
    int err = 0;
#pragma omp parallel
    {
        double *Bp = (double *)aligned_alloc(64, sizeof(double) * KC * NC);
        double *Ap = (double *)aligned_alloc(64, sizeof(double) * KC * MR);
        if (!Bp || !Ap) {
#pragma omp atomic write
            err = 1;
        }
#pragma omp barrier
        if (!err) {
#pragma omp for collapse(2) schedule(dynamic)
            for (int64_t jt = 0; jt < nct; ++jt) {
                for (int64_t rc = 0; rc < nrc; ++rc) {
                    int64_t j0 = jt * NC, jn = (n - j0 < NC) ? n - j0 : NC;
                    int64_t r0 = rc * MCH, r1 = (r0 + MCH < nrows) ? r0 + MCH : nrows;
                    for (int64_t p0 = 0; p0 < k; p0 += KC) {
                        int64_t pn = (k - p0 < KC) ? k - p0 : KC;
                        for (int64_t p = 0; p < pn; ++p)
                            for (int64_t j = 0; j < NC; ++j)
                                Bp[p * NC + j] = (j < jn) ? B[rsB[p0 + p] + csB[j0 + j]] : 0.0;
                        for (int64_t rt = r0; rt < r1; rt += MR) {
                            int64_t rn = (r1 - rt < MR) ? r1 - rt : MR;
                            for (int64_t p = 0; p < pn; ++p)
                                for (int64_t i = 0; i < MR; ++i) {
                                    int64_t row = (i < rn) ? (rows ? rows[rt + i] : rt + i) : -1;
                                    Ap[p * MR + i] = (row >= 0) ? A[rsA[row] + csA[p0 + p]] : 0.0;
                                }
                            for (int64_t jr = 0; jr < jn; jr += NR) {
                                double acc[MR][NR];
                                for (int i = 0; i < MR; ++i)
                                    for (int j = 0; j < NR; ++j)
                                        acc[i][j] = (i < rn && jr + j < jn) ? out[(rt + i) * n + j0 + jr + j] : 0.0;
                                for (int64_t p = 0; p < pn; ++p) {
                                    const double *a = Ap + p * MR, *b = Bp + p * NC + jr;
                                    for (int i = 0; i < MR; ++i)
                                        for (int j = 0; j < NR; ++j)
                                            acc[i][j] += a[i] * b[j];
                                }
                                for (int i = 0; i < rn; ++i)
                                    for (int j = 0; j < NR && jr + j < jn; ++j)
                                        out[(rt + i) * n + j0 + jr + j] = acc[i][j];
                            }
                        }
                    }
                    for (int64_t r = r0; r < r1; ++r) {
                        int64_t row = rows ? rows[r] : r;
                        for (int64_t j = j0; j < j0 + jn; ++j) {
                            double s = out[r * n + j];
                            out[r * n + j] = (beta == 0.0) ? alpha * s : alpha * s + beta * C0[rsC[row] + csC[j]];
                        }
                    }
                }
            }
        }
        free(Bp);
        free(Ap);
    }
    return err ? ORC_ERR_ALLOC : ORC_OK;
}

/* y[i] = sum_j T[rs[i] + cs[j]] * x[j]   (each y[i] is one running sum over j = 0..n-1 in order; rows are
 * processed in chunks so that the inner loop runs along the rows, which is the contiguous direction of the
 * column-major layouts used here) */
int orc_matvec(const double *T, const int64_t *rs, const int64_t *cs, int64_t m, int64_t n, const double *x, double *y)
{
    const int64_t CH = 512;
#pragma omp parallel for schedule(dynamic)
    for (int64_t i0 = 0; i0 < m; i0 += CH) {
        int64_t i1 = i0 + CH < m ? i0 + CH : m;
        for (int64_t i = i0; i < i1; ++i)
            y[i] = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            const double *col = T + cs[j];
            const double xj = x[j];
            for (int64_t i = i0; i < i1; ++i)
                y[i] += col[rs[i]] * xj;
        }
    }
    return ORC_OK;
}
