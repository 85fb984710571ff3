/*
 * CPU oracle for scaled dot-product attention (forward).  TEST INFRASTRUCTURE ONLY:
 * it exists to check the HIP path, shares no code with it, and must never be
 * called from the product path.
 *
 * What it computes is the plain definition of the paper's Eq. 1 (Section 3.1),
 * written out row by row in float64, with the mask M = 0 or, when `causal` is
 * set, the causal mask of Section 4.1.3 (M_ij = 0 for j <= i, -inf for j > i:
 * keys after the query contribute nothing), which simply shortens the sums to
 * j = 0..i:
 *
 *     s_ij  = scale * sum_d q_id * k_jd          (j = 0..S-1, or 0..i if causal)
 *     M_i   = max_j s_ij
 *     e_ij  = exp(s_ij - M_i)
 *     L_i   = sum_j e_ij
 *     O_id  = (sum_j e_ij * v_jd) / L_i
 *     LSE_i = M_i + ln L_i
 *
 * The full score row is materialised; there is no tiling, no online rescale and
 * no reordering beyond "subtract the row maximum before exponentiating", which
 * leaves the softmax unchanged.  The division by L_i is the paper's final
 * O_i = o_i / l_i of Section 4.1.2.
 *
 * Inputs are float32 arrays that hold FP16/BF16-rounded values exactly
 * (Section 4.1.3: inputs are FP16 or BF16); every operation promotes to double.
 *
 * Layout: q, k, v are contiguous [BH, S, D] (Section 4.1.1: [B,H,S,D] viewed as
 * [BH,S,D]).  `rows` selects query rows (same subset for every bh); NULL means
 * all S rows.  Outputs: o [BH, nrows, D] double, lse [BH, nrows] double
 * (nullable), p [BH, nrows, S] double (nullable; the softmax probabilities
 * e_ij / L_i, zero for masked keys, exposed for the rows-sum-to-one pin).
 *
 * sdpa_oracle_rows_kv is the same definition with Sq query rows against Skv
 * key/value rows (the KV-cache / decoding shapes of the paper's roadmap,
 * Section 8): q is [BH, Sq, D], k and v are [BH, Skv, D], and Eq. 1's score
 * matrix is Sq x Skv.  The paper defines the causal mask only for Sq = Skv;
 * the reading taken here is that the Sq queries are the LAST Sq positions of
 * the Skv-long sequence, so query row i sits at position i + (Skv - Sq) and
 * sees keys j <= i + (Skv - Sq).  Causal with Skv < Sq is rejected (its first
 * rows would see no key at all).
 *
 * Returns 0, or a negative number for bad arguments / allocation failure.
 */
#include <math.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int sdpa_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int sdpa_oracle_rows_kv(const float *q, const float *k, const float *v,
                        long BH, long Sq, long Skv, long D, double scale,
                        const long *rows, long nrows, int causal,
                        double *o, double *lse, double *p)
{
    if (!q || !k || !v || !o) return -1;
    if (BH < 0 || Sq < 0 || Skv < 0 || D <= 0) return -2;
    if (causal && Skv < Sq) return -2;
    if (!rows) nrows = Sq;
    if (nrows < 0) return -2;
    if (BH == 0 || Sq == 0 || nrows == 0) return 0;
    if (Skv == 0) return -2;                 /* a softmax over no keys is undefined */
    for (long r = 0; rows && r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= Sq) return -3;
    const long S = Skv;                      /* length of a score row */

    int failed = 0;
    const long total = BH * nrows;
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)S * sizeof(double));
        double *acc = (double *)malloc((size_t)D * sizeof(double));
        if (!s || !acc) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 4)
        for (long t = 0; t < total; ++t) {
            if (!s || !acc) continue;
            const long bh = t / nrows;
            const long r = t % nrows;
            const long i = rows ? rows[r] : r;
            const float *qi = q + (bh * Sq + i) * D;
            const float *kb = k + bh * Skv * D;
            const float *vb = v + bh * Skv * D;

            /* scores and their maximum; masked keys (after the query's position under the causal
               mask) are left out */
            const long J = causal ? i + (Skv - Sq) + 1 : Skv;
            double M = -INFINITY;
            for (long j = 0; j < J; ++j) {
                const float *kj = kb + j * D;
                double dot = 0.0;
                for (long d = 0; d < D; ++d) dot += (double)qi[d] * (double)kj[d];
                s[j] = scale * dot;
                if (s[j] > M) M = s[j];
            }
            /* exponentials, normaliser, weighted sum of value rows */
            double L = 0.0;
            for (long d = 0; d < D; ++d) acc[d] = 0.0;
            for (long j = 0; j < J; ++j) {
                const double e = exp(s[j] - M);
                s[j] = e;
                L += e;
                const float *vj = vb + j * D;
                for (long d = 0; d < D; ++d) acc[d] += e * (double)vj[d];
            }
            double *oi = o + t * D;
            for (long d = 0; d < D; ++d) oi[d] = acc[d] / L;
            if (lse) lse[t] = M + log(L);
            if (p) {
                double *pi = p + t * S;
                for (long j = 0; j < S; ++j) pi[j] = j < J ? s[j] / L : 0.0;
            }
        }
        free(s);
        free(acc);
    }
    return failed ? -4 : 0;
}

int sdpa_oracle_rows(const float *q, const float *k, const float *v,
                     long BH, long S, long D, double scale,
                     const long *rows, long nrows, int causal,
                     double *o, double *lse, double *p)
{
    return sdpa_oracle_rows_kv(q, k, v, BH, S, S, D, scale, rows, nrows, causal, o, lse, p);
}
