/*
 * mha_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, fp64 CPU statement of what one incremental decode step of
 * multi-head attention computes, written out from the definitions:
 *
 *   - scaled dot-product attention, Eq. 1:  Att(Q,K,V) = softmax(Q K^T / sqrt(d)) V
 *   - multi-head attention as a sum over heads, Eq. 2 / Eq. 6 (appendix B,
 *     with bias terms):  sum_i softmax(Q_i K_i^T / sqrt(d_k)) V_i W_i^O,
 *     Q_i = Q W_i^Q + b_i^Q,  K_i = H W_i^K + b_i^K,  V_i = H W_i^V + b_i^V.
 *   - the softmax scale is sqrt(d_k) (section 3.1: the normalisation factor
 *     is d_k, the rank of the expanded query, not d_m).
 *
 * mha_oracle()  is that definition: it projects K and V per head from the
 *               valid prefix of H and attends ("MHA without cache").  This is
 *               the function the GPU path is compared with.
 * el_oracle()   evaluates the same quantity in the order of Eq. 9 (expanded
 *               query against the unprojected H, key-bias term Q_i (b_i^K)^T
 *               kept inside the softmax, value-bias term sum_i b_i^V W_i^O
 *               added outside).  It exists only so the tests can check the
 *               losslessness identity Eq. 6 == Eq. 9 on the oracle itself.
 *
 * Readings of points the paper leaves open (the same list is in the design
 * notes of the repository):
 *   - an output-projection bias b^O is not in any equation; it is accepted
 *     (nullable) and added once per output row after the sum over heads.
 *   - padding: only positions t < lengths[b] exist.  Storage beyond the
 *     prefix is never read, so NaN/Inf there cannot influence the result.
 *   - lengths[b] must be >= 1 (with no position the softmax is undefined).
 *   - head i owns columns [i*d_k, (i+1)*d_k) of W^Q, W^K, W^V and rows
 *     [i*d_k, (i+1)*d_k) of W^O (the "concatenation" form of Eq. 2's footnote).
 *
 * Layout (all row-major, all double):
 *   H        [B, n, d_m]         hidden states (keys and values, H = K = V)
 *   lengths  [B] int32 or NULL   NULL means every row has length n
 *   Q        [B, beam, d_m]      one query per beam
 *   Wq,Wk,Wv [d_m, h*d_k]        used as x . W
 *   Wo       [h*d_k, d_m]
 *   bq,bk,bv [h*d_k] or NULL,  bo [d_m] or NULL
 *   out      [B, beam, d_m]
 *
 * No blocking, no fusion, no library calls beyond exp/sqrt.  OpenMP is used
 * over batch elements only (they are independent).  Nothing here is shared
 * with, included by, or derived from the HIP path.
 *
 * Parity pins (tests/test_oracle_pins.py): losslessness identity, key-bias
 * cancellation, value-bias pass-through, closed forms (len = 1, uniform
 * attention, arg-max limit), a hand-computed two-position example, a library
 * cross-check against torch's float64 multi_head_attention_forward, and
 * invariances.  No function in this file is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1
#define ORACLE_NO_MEM 2

static int check_args(int B, int beam, int n, int h, int d_m, int d_k,
                      const double *H, const int32_t *lengths, const double *Q,
                      const double *Wq, const double *Wk, const double *Wv,
                      const double *Wo, const double *out)
{
    if (B < 0 || beam < 1 || n < 1 || h < 1 || d_m < 1 || d_k < 1) return ORACLE_BAD_ARG;
    if (!H || !Q || !Wq || !Wk || !Wv || !Wo || !out) return ORACLE_BAD_ARG;
    if (lengths)
        for (int b = 0; b < B; ++b)
            if (lengths[b] < 1 || lengths[b] > n) return ORACLE_BAD_ARG;
    return ORACLE_OK;
}

/* y[c] = bias[c] + sum_k x[k] * W[k, c]   for c in [0, cols);  W is [rows, cols]. */
static void vec_times_mat(const double *x, const double *W, const double *bias,
                          int rows, int cols, double *y)
{
    for (int c = 0; c < cols; ++c) y[c] = bias ? bias[c] : 0.0;
    for (int k = 0; k < rows; ++k) {
        const double xk = x[k];
        const double *Wrow = W + (size_t)k * cols;
        for (int c = 0; c < cols; ++c) y[c] += xk * Wrow[c];
    }
}

/* In-place softmax over s[0..len): exp(s - max) / sum, Eq. 1's softmax. */
static void softmax_inplace(double *s, int len)
{
    double mx = s[0];
    for (int t = 1; t < len; ++t) if (s[t] > mx) mx = s[t];
    double sum = 0.0;
    for (int t = 0; t < len; ++t) { s[t] = exp(s[t] - mx); sum += s[t]; }
    for (int t = 0; t < len; ++t) s[t] /= sum;
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
 * Multi-head attention by its definition (Eq. 6 with Eq. 1): project keys and
 * values per head, score, softmax, weighted sum, output projection.
 */
int mha_oracle(int B, int beam, int n, int h, int d_m, int d_k,
               const double *H, const int32_t *lengths, const double *Q,
               const double *Wq, const double *bq, const double *Wk, const double *bk,
               const double *Wv, const double *bv, const double *Wo, const double *bo,
               double *out)
{
    int rc = check_args(B, beam, n, h, d_m, d_k, H, lengths, Q, Wq, Wk, Wv, Wo, out);
    if (rc) return rc;
    const int hd = h * d_k;
    const double inv_sqrt_dk = 1.0 / sqrt((double)d_k);
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int len = lengths ? lengths[b] : n;
        const double *Hb = H + (size_t)b * n * d_m;
        double *K = (double *)malloc((size_t)len * hd * sizeof(double));
        double *V = (double *)malloc((size_t)len * hd * sizeof(double));
        double *q = (double *)malloc((size_t)hd * sizeof(double));
        double *a = (double *)malloc((size_t)hd * sizeof(double));
        double *s = (double *)malloc((size_t)len * sizeof(double));
        if (!K || !V || !q || !a || !s) {
#pragma omp atomic write
            failed = 1;
        } else {
            /* K_i = H W_i^K + b_i^K and V_i = H W_i^V + b_i^V, all heads side by side. */
            for (int t = 0; t < len; ++t) {
                vec_times_mat(Hb + (size_t)t * d_m, Wk, bk, d_m, hd, K + (size_t)t * hd);
                vec_times_mat(Hb + (size_t)t * d_m, Wv, bv, d_m, hd, V + (size_t)t * hd);
            }
            for (int j = 0; j < beam; ++j) {
                const double *query = Q + ((size_t)b * beam + j) * d_m;
                double *o = out + ((size_t)b * beam + j) * d_m;
                /* Q_i = Q W_i^Q + b_i^Q, all heads side by side. */
                vec_times_mat(query, Wq, bq, d_m, hd, q);
                for (int i = 0; i < h; ++i) {
                    const double *qi = q + i * d_k;
                    for (int t = 0; t < len; ++t) {
                        const double *kt = K + (size_t)t * hd + i * d_k;
                        double dot = 0.0;
                        for (int c = 0; c < d_k; ++c) dot += qi[c] * kt[c];
                        s[t] = dot * inv_sqrt_dk;
                    }
                    softmax_inplace(s, len);
                    /* a_i = Prob_i V_i */
                    double *ai = a + i * d_k;
                    for (int c = 0; c < d_k; ++c) ai[c] = 0.0;
                    for (int t = 0; t < len; ++t) {
                        const double *vt = V + (size_t)t * hd + i * d_k;
                        for (int c = 0; c < d_k; ++c) ai[c] += s[t] * vt[c];
                    }
                }
                /* sum_i a_i W_i^O (+ b^O): the heads' rows of W^O are stacked, so
                   this is one vector-matrix product over the concatenated a. */
                vec_times_mat(a, Wo, bo, hd, d_m, o);
            }
        }
        free(K); free(V); free(q); free(a); free(s);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}

/*
 * The same quantity evaluated in the order of Eq. 9: per head, expand the
 * query to model dimension (Eq. 7: FFN_i^Q(Q) = (Q W_i^Q + b_i^Q)(W_i^K)^T),
 * score it against the unprojected H, keep the key-bias term Q_i (b_i^K)^T
 * inside the softmax, take X = Prob_i . H, apply FFN_i^O(X) = X W_i^V W_i^O
 * (Eq. 8) and add sum_i b_i^V W_i^O.
 */
int el_oracle(int B, int beam, int n, int h, int d_m, int d_k,
              const double *H, const int32_t *lengths, const double *Q,
              const double *Wq, const double *bq, const double *Wk, const double *bk,
              const double *Wv, const double *bv, const double *Wo, const double *bo,
              double *out)
{
    int rc = check_args(B, beam, n, h, d_m, d_k, H, lengths, Q, Wq, Wk, Wv, Wo, out);
    if (rc) return rc;
    const int hd = h * d_k;
    const double inv_sqrt_dk = 1.0 / sqrt((double)d_k);
    int failed = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        const int len = lengths ? lengths[b] : n;
        const double *Hb = H + (size_t)b * n * d_m;
        double *q = (double *)malloc((size_t)hd * sizeof(double));
        double *elq = (double *)malloc((size_t)d_m * sizeof(double));
        double *X = (double *)malloc((size_t)d_m * sizeof(double));
        double *xv = (double *)malloc((size_t)d_k * sizeof(double));
        double *s = (double *)malloc((size_t)len * sizeof(double));
        if (!q || !elq || !X || !xv || !s) {
#pragma omp atomic write
            failed = 1;
        } else {
            for (int j = 0; j < beam; ++j) {
                const double *query = Q + ((size_t)b * beam + j) * d_m;
                double *o = out + ((size_t)b * beam + j) * d_m;
                for (int d = 0; d < d_m; ++d) o[d] = bo ? bo[d] : 0.0;
                vec_times_mat(query, Wq, bq, d_m, hd, q);
                for (int i = 0; i < h; ++i) {
                    const double *qi = q + i * d_k;
                    /* EL-Q_i[d] = sum_c Q_i[c] W^K[d, i*d_k + c] */
                    for (int d = 0; d < d_m; ++d) {
                        double acc = 0.0;
                        for (int c = 0; c < d_k; ++c) acc += qi[c] * Wk[(size_t)d * hd + i * d_k + c];
                        elq[d] = acc;
                    }
                    /* Q_i (b_i^K)^T : one scalar, the same for every position. */
                    double qbk = 0.0;
                    if (bk) for (int c = 0; c < d_k; ++c) qbk += qi[c] * bk[i * d_k + c];
                    for (int t = 0; t < len; ++t) {
                        const double *ht = Hb + (size_t)t * d_m;
                        double dot = 0.0;
                        for (int d = 0; d < d_m; ++d) dot += elq[d] * ht[d];
                        s[t] = (dot + qbk) * inv_sqrt_dk;
                    }
                    softmax_inplace(s, len);
                    /* X = Prob_i . H */
                    for (int d = 0; d < d_m; ++d) X[d] = 0.0;
                    for (int t = 0; t < len; ++t) {
                        const double *ht = Hb + (size_t)t * d_m;
                        for (int d = 0; d < d_m; ++d) X[d] += s[t] * ht[d];
                    }
                    /* FFN_i^O(X) + b_i^V W_i^O = (X W_i^V + b_i^V) W_i^O */
                    for (int c = 0; c < d_k; ++c) {
                        double acc = bv ? bv[i * d_k + c] : 0.0;
                        for (int d = 0; d < d_m; ++d) acc += X[d] * Wv[(size_t)d * hd + i * d_k + c];
                        xv[c] = acc;
                    }
                    for (int c = 0; c < d_k; ++c) {
                        const double *Worow = Wo + (size_t)(i * d_k + c) * d_m;
                        for (int d = 0; d < d_m; ++d) o[d] += xv[c] * Worow[d];
                    }
                }
            }
        }
        free(q); free(elq); free(X); free(xv); free(s);
    }
    return failed ? ORACLE_NO_MEM : ORACLE_OK;
}
