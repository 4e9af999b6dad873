/*
 * fp64 CPU oracle for causal softmax attention and its analytic gradients.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call into this
 * file; it exists so that the HIP kernels can be compared element by element
 * with the plain definition of what the chunked method computes.  It shares
 * no code, header, table or helper with the GPU library.
 *
 * What it follows: the paper's distributed attention (Sec. 4.1) is a pure
 * re-scheduling of ordinary causal attention -- a query never attends a later
 * key (Sec. 4.2), the diagonal is included, and the result must not differ
 * from unchunked training (App. A).  So the oracle is the textbook definition
 * written out, one query row (or one key column) at a time, two-pass softmax,
 * no blocking, no online rescaling:
 *
 *   s_ij  = scale * sum_d Q[i,h,d] K[j,kv(h),d]          j <= i
 *   LSE_i = m_i + log sum_j exp(s_ij - m_i),  m_i = max_j s_ij
 *   p_ij  = exp(s_ij - LSE_i)
 *   O_i   = sum_j p_ij V[j,kv(h),:]
 *   Delta_i = sum_d dO[i,h,d] O[i,h,d]
 *   dP_ij = sum_d dO[i,h,d] V[j,kv(h),d]
 *   dS_ij = p_ij (dP_ij - Delta_i)
 *   dQ_i  = scale * sum_j dS_ij K[j,kv(h),:]
 *   dK_j  = scale * sum_{h in group} sum_{i>=j} dS_ij Q[i,h,:]
 *   dV_j  =         sum_{h in group} sum_{i>=j} p_ij  dO[i,h,:]
 *
 * kv(h) = h / (Hq/Hkv) (grouped-query head sharing; the gradient of a shared
 * K/V head is the sum over the query heads that read it).
 *
 * Layout: tensors are row-major [rows, heads, D]; per-row scalars are
 * [rows, Hq].  Everything is double.
 *
 * Block-sparse variant (Sec. 5.5: with sparse attention only part of the key /
 * value chunks is fetched, the queries are always the whole sequence).  The
 * sequence is cut into chunks of `chunk` rows and a u x u byte matrix says
 * which key chunks a query chunk reads: key j is allowed for query i iff
 * j <= i and mask[(i / chunk) * u + j / chunk] != 0.  Every sum over j above
 * (and over i for dK, dV) then runs over the allowed pairs only; nothing else
 * changes.  mask == NULL is the dense definition.  The diagonal entries of the
 * mask must be set, so that every query row keeps at least its own key.
 *
 * Two entry points: a row evaluator (everything that is indexed by a query
 * row) and a column evaluator (everything indexed by a key row).  The full
 * problem is "all rows, then all columns"; sampled checks at large S call the
 * same two functions on a subset of rows / a tail window of columns.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int fpdt_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double dot(const double *a, const double *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int d = 0; d < n; ++d) acc += a[d] * b[d];
    return acc;
}

/*
 * Row evaluator.  For each listed query row rows[r] (global index in [0,S))
 * and every query head: O, LSE and, when dOr != NULL, Delta and dQ.
 *
 *   Qr, dOr : [n, Hq, D]   the listed rows of Q and dO (gathered by caller)
 *   K, V    : [S, Hkv, D]  the whole key / value tensors
 *   O, dQ   : [n, Hq, D]   out
 *   LSE, Delta : [n, Hq]   out
 * Returns 0, or 1 on bad arguments / allocation failure.
 */
/* key j allowed for query i (j <= i is the caller's loop bound) */
static int allowed(const uint8_t *mask, int64_t chunk, int64_t u, int64_t i, int64_t j)
{
    return !mask || mask[(i / chunk) * u + j / chunk] != 0;
}

static int mask_ok(const uint8_t *mask, int64_t chunk, int64_t S)
{
    if (!mask) return 1;
    if (chunk <= 0 || S % chunk != 0) return 0;
    const int64_t u = S / chunk;
    for (int64_t m = 0; m < u; ++m)
        if (!mask[m * u + m]) return 0;
    return 1;
}

int fpdt_oracle_rows_blocksparse(const double *Qr, const double *dOr, const int64_t *rows, int64_t n,
                                 const double *K, const double *V, int64_t S, int Hq, int Hkv,
                                 int D, double scale, int64_t chunk, const uint8_t *mask,
                                 double *O, double *LSE, double *Delta, double *dQ)
{
    if (!Qr || !rows || !K || !V || !O || !LSE || n < 0 || S <= 0 || Hq <= 0 || Hkv <= 0 ||
        D <= 0 || Hq % Hkv != 0 || !mask_ok(mask, chunk, S))
        return 1;
    const int64_t u = mask ? S / chunk : 1;
    if (dOr && (!Delta || !dQ)) return 1;
    for (int64_t r = 0; r < n; ++r)
        if (rows[r] < 0 || rows[r] >= S) return 1;
    const int g = Hq / Hkv;
    int fail = 0;
#pragma omp parallel
    {
        double *p = (double *)malloc(sizeof(double) * (size_t)S);
        if (!p) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp barrier
        if (!fail) {
#pragma omp for collapse(2) schedule(dynamic, 1)
            for (int64_t r = 0; r < n; ++r) {
                for (int h = 0; h < Hq; ++h) {
                    const int64_t i = rows[r];
                    const int kv = h / g;
                    const double *q = Qr + ((size_t)r * Hq + h) * D;
                    double *o = O + ((size_t)r * Hq + h) * D;
                    /* scores of the allowed keys j <= i, and their maximum */
                    double m = -INFINITY;
                    for (int64_t j = 0; j <= i; ++j) {
                        if (!allowed(mask, chunk, u, i, j)) continue;
                        p[j] = scale * dot(q, K + ((size_t)j * Hkv + kv) * D, D);
                        if (p[j] > m) m = p[j];
                    }
                    double l = 0.0;
                    for (int64_t j = 0; j <= i; ++j)
                        if (allowed(mask, chunk, u, i, j)) l += exp(p[j] - m);
                    const double lse = m + log(l);
                    LSE[(size_t)r * Hq + h] = lse;
                    for (int d = 0; d < D; ++d) o[d] = 0.0;
                    for (int64_t j = 0; j <= i; ++j) {
                        if (!allowed(mask, chunk, u, i, j)) continue;
                        p[j] = exp(p[j] - lse); /* probabilities from here on */
                        const double *v = V + ((size_t)j * Hkv + kv) * D;
                        const double pj = p[j];
                        for (int d = 0; d < D; ++d) o[d] += pj * v[d];
                    }
                    if (!dOr) continue;
                    const double *go = dOr + ((size_t)r * Hq + h) * D;
                    double *gq = dQ + ((size_t)r * Hq + h) * D;
                    const double delta = dot(go, o, D);
                    Delta[(size_t)r * Hq + h] = delta;
                    for (int d = 0; d < D; ++d) gq[d] = 0.0;
                    for (int64_t j = 0; j <= i; ++j) {
                        if (!allowed(mask, chunk, u, i, j)) continue;
                        const double dp = dot(go, V + ((size_t)j * Hkv + kv) * D, D);
                        const double ds = p[j] * (dp - delta);
                        const double *k = K + ((size_t)j * Hkv + kv) * D;
                        for (int d = 0; d < D; ++d) gq[d] += ds * k[d];
                    }
                    for (int d = 0; d < D; ++d) gq[d] *= scale;
                }
            }
        }
        free(p);
    }
    return fail;
}

int fpdt_oracle_rows(const double *Qr, const double *dOr, const int64_t *rows, int64_t n,
                     const double *K, const double *V, int64_t S, int Hq, int Hkv, int D,
                     double scale, double *O, double *LSE, double *Delta, double *dQ)
{
    return fpdt_oracle_rows_blocksparse(Qr, dOr, rows, n, K, V, S, Hq, Hkv, D, scale, 0, NULL, O,
                                        LSE, Delta, dQ);
}

/*
 * Column evaluator.  For each listed key row cols[c] and every KV head: dK
 * and dV, summed over the query heads of the group and over all query rows
 * i >= cols[c].
 *
 *   Q, dO      : [S - row_base, Hq, D]  query rows row_base .. S-1
 *   LSE, Delta : [S - row_base, Hq]     the same rows (from the row evaluator)
 *   Kc, Vc     : [n, Hkv, D]            the listed key rows of K and V
 *   dK, dV     : [n, Hkv, D]            out
 * Every cols[c] must be >= row_base: query rows before a column never attend
 * it, so a row window that starts at or before the smallest listed column
 * holds every contribution.
 */
int fpdt_oracle_cols_blocksparse(const double *Q, const double *dO, const double *LSE,
                                 const double *Delta, int64_t row_base, const double *Kc,
                                 const double *Vc, const int64_t *cols, int64_t n, int64_t S, int Hq,
                                 int Hkv, int D, double scale, int64_t chunk, const uint8_t *mask,
                                 double *dK, double *dV)
{
    if (!Q || !dO || !LSE || !Delta || !Kc || !Vc || !cols || !dK || !dV || n < 0 || S <= 0 ||
        Hq <= 0 || Hkv <= 0 || D <= 0 || Hq % Hkv != 0 || row_base < 0 || row_base >= S ||
        !mask_ok(mask, chunk, S))
        return 1;
    const int64_t u = mask ? S / chunk : 1;
    for (int64_t c = 0; c < n; ++c)
        if (cols[c] < row_base || cols[c] >= S) return 1;
    const int g = Hq / Hkv;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t c = 0; c < n; ++c) {
        for (int kv = 0; kv < Hkv; ++kv) {
            const int64_t j = cols[c];
            const double *k = Kc + ((size_t)c * Hkv + kv) * D;
            const double *v = Vc + ((size_t)c * Hkv + kv) * D;
            double *gk = dK + ((size_t)c * Hkv + kv) * D;
            double *gv = dV + ((size_t)c * Hkv + kv) * D;
            for (int d = 0; d < D; ++d) gk[d] = gv[d] = 0.0;
            for (int h = kv * g; h < (kv + 1) * g; ++h) {
                for (int64_t i = j; i < S; ++i) {
                    if (!allowed(mask, chunk, u, i, j)) continue;
                    const size_t ri = (size_t)(i - row_base);
                    const double *q = Q + (ri * Hq + h) * D;
                    const double *go = dO + (ri * Hq + h) * D;
                    const double s = scale * dot(q, k, D);
                    const double p = exp(s - LSE[ri * Hq + h]);
                    const double dp = dot(go, v, D);
                    const double ds = p * (dp - Delta[ri * Hq + h]);
                    for (int d = 0; d < D; ++d) {
                        gk[d] += ds * q[d];
                        gv[d] += p * go[d];
                    }
                }
            }
            for (int d = 0; d < D; ++d) gk[d] *= scale;
        }
    }
    return 0;
}

int fpdt_oracle_cols(const double *Q, const double *dO, const double *LSE, const double *Delta,
                     int64_t row_base, const double *Kc, const double *Vc, const int64_t *cols,
                     int64_t n, int64_t S, int Hq, int Hkv, int D, double scale, double *dK,
                     double *dV)
{
    return fpdt_oracle_cols_blocksparse(Q, dO, LSE, Delta, row_base, Kc, Vc, cols, n, S, Hq, Hkv, D,
                                        scale, 0, NULL, dK, dV);
}
