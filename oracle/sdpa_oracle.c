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
 * Section 7): q is [BH, Sq, D], k and v are [BH, Skv, D], and Eq. 1's score
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

/*
 * Backward pass (the paper's roadmap, Section 7, names it as future work and prints no formula):
 * the gradient of the scalar  Lambda = sum_{i,d} dO_id * O_id  with O from Eq. 1 (Section 3.1),
 * with respect to Q, K and V, written out row by row in float64.  Differentiating Eq. 1
 * (P = row softmax of the scaled, masked scores, O = P V):
 *
 *     dV_jd = sum_i P_ij dO_id
 *     dP_ij = sum_d dO_id V_jd
 *     dS_ij = P_ij (dP_ij - sum_j' P_ij' dP_ij')        (Jacobian of the row softmax)
 *     dQ_id = scale * sum_j dS_ij K_jd
 *     dK_jd = scale * sum_i dS_ij Q_id
 *
 * Masked keys (j > i under the causal mask of Section 4.1.3) have P_ij = 0 and drop out of every sum.
 * Pass 1 walks query rows (P_i, dP_i, the inner sum, dQ_i; keeps M_i, L_i and the inner sum), pass 2
 * walks key rows and recomputes P_ij = exp(s_ij - M_i) / L_i for every query i.  Nothing is tiled.
 *
 * q, k, v, dout: float32 [BH, S, D] holding 16-bit-rounded values exactly.  qrows / krows select the
 * rows for which dQ / (dK, dV) are produced (NULL = all S): dq is [BH, nq, D], dk and dv are
 * [BH, nk, D], all double.  Returns 0 or a negative error as sdpa_oracle_rows does.
 */
int sdpa_oracle_bwd(const float *q, const float *k, const float *v, const float *dout,
                    long BH, long S, long D, double scale, int causal,
                    const long *qrows, long nq, const long *krows, long nk,
                    double *dq, double *dk, double *dv)
{
    if (!q || !k || !v || !dout || !dq || !dk || !dv) return -1;
    if (BH < 0 || S < 0 || D <= 0) return -2;
    if (!qrows) nq = S;
    if (!krows) nk = S;
    if (nq < 0 || nk < 0) return -2;
    if (BH == 0 || S == 0) return 0;
    for (long r = 0; qrows && r < nq; ++r) if (qrows[r] < 0 || qrows[r] >= S) return -3;
    for (long r = 0; krows && r < nk; ++r) if (krows[r] < 0 || krows[r] >= S) return -3;

    /* per query row: maximum M, normaliser L and inner = sum_j P_ij dP_ij */
    double *Mx = (double *)malloc((size_t)BH * S * sizeof(double));
    double *Lx = (double *)malloc((size_t)BH * S * sizeof(double));
    double *In = (double *)malloc((size_t)BH * S * sizeof(double));
    long *qslot = (long *)malloc((size_t)S * sizeof(long));   /* row -> position in qrows, or -1 */
    if (!Mx || !Lx || !In || !qslot) { free(Mx); free(Lx); free(In); free(qslot); return -4; }
    for (long i = 0; i < S; ++i) qslot[i] = qrows ? -1 : i;
    for (long r = 0; qrows && r < nq; ++r) qslot[qrows[r]] = r;

    int failed = 0;
#pragma omp parallel
    {
        double *p = (double *)malloc((size_t)S * sizeof(double));
        double *dp = (double *)malloc((size_t)S * sizeof(double));
        if (!p || !dp) {
#pragma omp atomic write
            failed = 1;
        }
        /* pass 1: query rows */
#pragma omp for schedule(dynamic, 4)
        for (long t = 0; t < BH * S; ++t) {
            if (!p || !dp) continue;
            const long bh = t / S, i = t % S;
            const float *qi = q + (bh * S + i) * D, *doi = dout + (bh * S + i) * D;
            const float *kb = k + bh * S * D, *vb = v + bh * S * D;
            const long J = causal ? i + 1 : S;
            double M = -INFINITY;
            for (long j = 0; j < J; ++j) {
                double dot = 0.0, dd = 0.0;
                for (long d = 0; d < D; ++d) {
                    dot += (double)qi[d] * (double)kb[j * D + d];
                    dd += (double)doi[d] * (double)vb[j * D + d];
                }
                p[j] = scale * dot;
                dp[j] = dd;
                if (p[j] > M) M = p[j];
            }
            double L = 0.0;
            for (long j = 0; j < J; ++j) { p[j] = exp(p[j] - M); L += p[j]; }
            double inner = 0.0;
            for (long j = 0; j < J; ++j) { p[j] /= L; inner += p[j] * dp[j]; }
            Mx[t] = M; Lx[t] = L; In[t] = inner;
            if (qslot[i] >= 0) {
                double *dqi = dq + (bh * nq + qslot[i]) * D;
                for (long d = 0; d < D; ++d) dqi[d] = 0.0;
                for (long j = 0; j < J; ++j) {
                    const double ds = p[j] * (dp[j] - inner);
                    for (long d = 0; d < D; ++d) dqi[d] += ds * (double)kb[j * D + d];
                }
                for (long d = 0; d < D; ++d) dqi[d] *= scale;
            }
        }
        /* pass 2: key rows (the implicit barrier of the loop above has made M, L, inner visible) */
#pragma omp for schedule(dynamic, 4)
        for (long t = 0; t < BH * nk; ++t) {
            const long bh = t / nk, r = t % nk;
            const long j = krows ? krows[r] : r;
            const float *kj = k + (bh * S + j) * D, *vj = v + (bh * S + j) * D;
            double *dkj = dk + t * D, *dvj = dv + t * D;
            for (long d = 0; d < D; ++d) { dkj[d] = 0.0; dvj[d] = 0.0; }
            for (long i = causal ? j : 0; i < S; ++i) {     /* queries that see key j */
                const float *qi = q + (bh * S + i) * D, *doi = dout + (bh * S + i) * D;
                double dot = 0.0, dd = 0.0;
                for (long d = 0; d < D; ++d) {
                    dot += (double)qi[d] * (double)kj[d];
                    dd += (double)doi[d] * (double)vj[d];
                }
                const double pij = exp(scale * dot - Mx[bh * S + i]) / Lx[bh * S + i];
                const double ds = pij * (dd - In[bh * S + i]);
                for (long d = 0; d < D; ++d) {
                    dkj[d] += ds * (double)qi[d];
                    dvj[d] += pij * (double)doi[d];
                }
            }
            for (long d = 0; d < D; ++d) dkj[d] *= scale;
        }
        free(p);
        free(dp);
    }
    free(Mx); free(Lx); free(In); free(qslot);
    return failed ? -4 : 0;
}
