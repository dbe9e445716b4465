/*
 * CPU oracle for the InfLLM-V2 dense-sparse switchable attention path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * method computes, written from the paper (arXiv 2509.24663).  Only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the GPU library
 * shares no code with it and never calls it.
 *
 * Conventions: inputs and outputs are float32 arrays (bf16 workloads pass
 * bf16-exact float32 values); every sum, dot product, exponential and
 * normalisation is carried out in double and rounded to float32 once, on store.
 * Softmax is the textbook three-step form (max, exp, divide): no tiling, no
 * online rescaling, no fusion.  All indices are 0-based; token t lies in block
 * t / B.  One call handles one KV head of one sequence; `pos[r]` is the token
 * position of query row r (so a decode step is the single row pos = L-1, and a
 * sample of rows of a long prefill costs only those rows).
 *
 * Readings of the paper where it is silent (all restated in the design notes):
 *   - attention is causal (keys u <= t);
 *   - one softmax scale (1/sqrt(d_h) by default) multiplies the logits both in
 *     the compressed-key scores (Eq. 4) and in the attention itself (Eq. 1);
 *   - compressed key i covers tokens [i*s, i*s + l) and exists only if the whole
 *     window lies inside the sequence; query t sees key i only if the window
 *     ends at or before t;
 *   - rows with no visible compressed key have all-zero scores;
 *   - the top-k budget is min(N_topk, #remaining blocks), ties go to the
 *     smaller block index;
 *   - LSE Approximation (Sec. 3.4, Eq. 7, Alg. 1): the first pass of Alg. 1 runs
 *     over K^{C2} (window 4 l_C1, stride 4 s_C1, same visibility rule) and its
 *     log-sum-exp is used as printed, with no correction for the 4x smaller key
 *     count; a row that sees no K^{C2} key has all-zero scores.
 *
 * Parity pins (tests/test_oracle_*.py): closed forms for the mean pooling,
 * softmax rows summing to G, brute-force masked dense attention, sparse == dense
 * when every block is kept, library softmax / SDPA cross-checks, a full-sort
 * brute-force top-k, decode == last prefill row; for the gradients of stage 4
 * (oracle_attn_bwd): automatic differentiation of textbook masked attention in
 * float64, central differences, and the column sums of dV.  The choice of which compressed
 * keys are visible and the pooling-window alignment are fixed by this file, not
 * by any printed value in the paper: for those two conventions parity is
 * unpinned by the paper itself.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* number of complete compression windows in a sequence of n tokens (Sec. 3.3, Eq. 3) */
int oracle_num_cmp(int n, int lc, int sc) { return n < lc ? 0 : (n - lc) / sc + 1; }

/* number of compressed keys whose window ends at or before token t */
static int visible_cmp(int t, int lc, int sc) { return t < lc - 1 ? 0 : (t - lc + 1) / sc + 1; }

int oracle_visible_cmp(int t, int lc, int sc) { return visible_cmp(t, lc, sc); }

/* Stage 1, Eq. 3:  kc[i] = mean of K rows [i*sc, i*sc + lc).   K [n][d] -> kc [nc][d] */
void oracle_compress_k(const float *K, int n, int d, int lc, int sc, float *kc) {
    int nc = oracle_num_cmp(n, lc, sc);
#pragma omp parallel for schedule(static)
    for (int i = 0; i < nc; ++i) {
        for (int c = 0; c < d; ++c) {
            double s = 0.0;
            for (int u = 0; u < lc; ++u) s += (double)K[(size_t)(i * sc + u) * d + c];
            kc[(size_t)i * d + c] = (float)(s / (double)lc);
        }
    }
}

/* Stage 2, Eq. 4 + Eq. 5: per query head a softmax over the visible compressed keys,
 * then the sum of the G per-head probability rows.
 * Q [nr][G][d], kc [nc][d]  ->  shared [nr][row_stride] (entries >= vis(t) are zero). */
void oracle_block_scores(const float *Q, const int32_t *pos, int nr, int G, int d, const float *kc, int nc,
                         int lc, int sc, double scale, float *shared, int64_t row_stride) {
#pragma omp parallel
    {
        double *z = (double *)malloc(sizeof(double) * (size_t)(nc > 0 ? nc : 1));
        double *acc = (double *)malloc(sizeof(double) * (size_t)(nc > 0 ? nc : 1));
#pragma omp for schedule(dynamic, 16)
        for (int r = 0; r < nr; ++r) {
            int v = visible_cmp(pos[r], lc, sc);
            if (v > nc) v = nc;
            float *out = shared + (size_t)r * row_stride;
            for (int i = 0; i < nc; ++i) out[i] = 0.0f;
            if (v == 0) continue;
            for (int i = 0; i < v; ++i) acc[i] = 0.0;
            for (int g = 0; g < G; ++g) {
                const float *q = Q + ((size_t)r * G + g) * d;
                double zmax = -INFINITY;
                for (int i = 0; i < v; ++i) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)kc[(size_t)i * d + c];
                    z[i] = scale * dot;
                    if (z[i] > zmax) zmax = z[i];
                }
                double den = 0.0;
                for (int i = 0; i < v; ++i) {
                    z[i] = exp(z[i] - zmax);
                    den += z[i];
                }
                for (int i = 0; i < v; ++i) acc[i] += z[i] / den;
            }
            for (int i = 0; i < v; ++i) out[i] = (float)acc[i];
        }
        free(z);
        free(acc);
    }
}

/* Stage 2 with LSE Approximation, Sec. 3.4 Eq. 7 and Alg. 1: the log-sum-exp of every (row, head) is taken
 * over the coarse keys kc2 (first pass), the fine scores exp(z_i - lse) over kc (second pass) are summed
 * over the G heads.   kc [nc][d] with (lc, sc), kc2 [nc2][d] with (lc2, sc2). */
void oracle_block_scores_lse_approx(const float *Q, const int32_t *pos, int nr, int G, int d, const float *kc,
                                    int nc, int lc, int sc, const float *kc2, int nc2, int lc2, int sc2,
                                    double scale, float *shared, int64_t row_stride) {
#pragma omp parallel
    {
        double *acc = (double *)malloc(sizeof(double) * (size_t)(nc > 0 ? nc : 1));
        double *z2 = (double *)malloc(sizeof(double) * (size_t)(nc2 > 0 ? nc2 : 1));
#pragma omp for schedule(dynamic, 16)
        for (int r = 0; r < nr; ++r) {
            int v = visible_cmp(pos[r], lc, sc);
            int v2 = visible_cmp(pos[r], lc2, sc2);
            if (v > nc) v = nc;
            if (v2 > nc2) v2 = nc2;
            float *out = shared + (size_t)r * row_stride;
            for (int i = 0; i < nc; ++i) out[i] = 0.0f;
            if (v == 0 || v2 == 0) continue;
            for (int i = 0; i < v; ++i) acc[i] = 0.0;
            for (int g = 0; g < G; ++g) {
                const float *q = Q + ((size_t)r * G + g) * d;
                /* first pass: lse over the coarse keys */
                double zmax = -INFINITY;
                for (int i = 0; i < v2; ++i) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)kc2[(size_t)i * d + c];
                    z2[i] = scale * dot;
                    if (z2[i] > zmax) zmax = z2[i];
                }
                double den = 0.0;
                for (int i = 0; i < v2; ++i) den += exp(z2[i] - zmax);
                double lse = zmax + log(den);
                /* second pass: fine scores normalised with it */
                for (int i = 0; i < v; ++i) {
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)kc[(size_t)i * d + c];
                    acc[i] += exp(scale * dot - lse);
                }
            }
            for (int i = 0; i < v; ++i) out[i] = (float)acc[i];
        }
        free(acc);
        free(z2);
    }
}

/* Stage 3, Eq. 6 + Eq. 2: max-pool the shared scores to one value per selection block,
 * force the initial and local blocks, take the top-k of the rest.
 * shared [nr][row_stride] -> idx [nr][topk_total] ascending, padded with -1.
 * cmp_out (may be NULL) [nr][cmp_stride] receives the pooled scores of blocks 0..b_t. */
void oracle_topk_blocks(const float *shared, int64_t row_stride, const int32_t *pos, int nr, int lc, int sc,
                        int B, int pool_len, int pool_stride, int pool_pad, int n_init, int n_local,
                        int topk_total, int32_t *idx, float *cmp_out, int64_t cmp_stride) {
    int n_topk = topk_total - n_init - n_local;
#pragma omp parallel for schedule(dynamic, 16)
    for (int r = 0; r < nr; ++r) {
        int t = pos[r];
        int bt = t / B;
        int v = visible_cmp(t, lc, sc);
        const float *row = shared + (size_t)r * row_stride;
        int nblk = bt + 1;
        float *cmp = (float *)malloc(sizeof(float) * (size_t)nblk);
        char *forced = (char *)calloc((size_t)nblk, 1);
        char *chosen = (char *)calloc((size_t)nblk, 1);
        for (int j = 0; j < nblk; ++j) {
            float m = 0.0f; /* empty window -> 0 (scores are never negative) */
            int lo = pool_stride * j - pool_pad, hi = lo + pool_len;
            for (int i = lo; i < hi; ++i)
                if (i >= 0 && i < v && row[i] > m) m = row[i];
            cmp[j] = m;
        }
        for (int j = 0; j < n_init && j < nblk; ++j) forced[j] = 1;
        for (int j = bt - n_local + 1; j <= bt; ++j)
            if (j >= 0) forced[j] = 1;
        int remaining = 0;
        for (int j = 0; j < nblk; ++j) {
            chosen[j] = forced[j];
            if (!forced[j]) ++remaining;
        }
        int kr = n_topk < remaining ? n_topk : remaining;
        for (int s = 0; s < kr; ++s) { /* repeated arg-max, first (smallest) index wins a tie */
            int best = -1;
            for (int j = 0; j < nblk; ++j)
                if (!chosen[j] && (best < 0 || cmp[j] > cmp[best])) best = j;
            chosen[best] = 1;
        }
        int32_t *o = idx + (size_t)r * topk_total;
        int w = 0;
        for (int j = 0; j < nblk; ++j)
            if (chosen[j]) o[w++] = j;
        for (; w < topk_total; ++w) o[w] = -1;
        if (cmp_out) {
            float *co = cmp_out + (size_t)r * cmp_stride;
            for (int j = 0; j < nblk; ++j) co[j] = cmp[j];
        }
        free(cmp);
        free(forced);
        free(chosen);
    }
}

/* exact softmax attention of one query row over an explicit list of key positions */
static void attend_row(const float *Qr, int G, int d, const float *K, const float *V, const int *keys,
                       int nk, double scale, float *Or, float *lser, double *z, double *o) {
    for (int g = 0; g < G; ++g) {
        const float *q = Qr + (size_t)g * d;
        double zmax = -INFINITY;
        for (int a = 0; a < nk; ++a) {
            const float *kr = K + (size_t)keys[a] * d;
            double dot = 0.0;
            for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)kr[c];
            z[a] = scale * dot;
            if (z[a] > zmax) zmax = z[a];
        }
        double den = 0.0;
        for (int a = 0; a < nk; ++a) {
            z[a] = exp(z[a] - zmax);
            den += z[a];
        }
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        for (int a = 0; a < nk; ++a) {
            double p = z[a] / den;
            const float *vr = V + (size_t)keys[a] * d;
            for (int c = 0; c < d; ++c) o[c] += p * (double)vr[c];
        }
        for (int c = 0; c < d; ++c) Or[(size_t)g * d + c] = (float)o[c];
        lser[g] = (float)(zmax + log(den));
    }
}

/* Stage 4, Appendix Alg. 2 stated directly: token t attends to the keys u <= t that lie in
 * one of its selected blocks.  Q [nr][G][d], K,V [n][d], idx [nr][topk_total]
 *   -> O [nr][G][d], lse [nr][G] (natural log of the softmax denominator incl. the max). */
void oracle_sparse_attn(const float *Q, const int32_t *pos, int nr, int G, int d, const float *K,
                        const float *V, int n, int B, const int32_t *idx, int topk_total, double scale,
                        float *O, float *lse) {
#pragma omp parallel
    {
        int cap = topk_total * B;
        int *keys = (int *)malloc(sizeof(int) * (size_t)cap);
        double *z = (double *)malloc(sizeof(double) * (size_t)cap);
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 16)
        for (int r = 0; r < nr; ++r) {
            int t = pos[r];
            int nk = 0;
            for (int s = 0; s < topk_total; ++s) {
                int j = idx[(size_t)r * topk_total + s];
                if (j < 0) continue;
                for (int u = j * B; u < (j + 1) * B && u <= t && u < n; ++u) keys[nk++] = u;
            }
            attend_row(Q + (size_t)r * G * d, G, d, K, V, keys, nk, scale, O + (size_t)r * G * d,
                       lse + (size_t)r * G, z, o);
        }
        free(keys);
        free(z);
        free(o);
    }
}

/* Dense causal GQA attention, Eq. 1 (Appendix Alg. 3 computes the same thing tile by tile). */
void oracle_dense_attn(const float *Q, const int32_t *pos, int nr, int G, int d, const float *K,
                       const float *V, int n, double scale, float *O, float *lse) {
#pragma omp parallel
    {
        int *keys = (int *)malloc(sizeof(int) * (size_t)(n > 0 ? n : 1));
        double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        double *o = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(dynamic, 4)
        for (int r = 0; r < nr; ++r) {
            int t = pos[r];
            int nk = 0;
            for (int u = 0; u <= t && u < n; ++u) keys[nk++] = u;
            attend_row(Q + (size_t)r * G * d, G, d, K, V, keys, nk, scale, O + (size_t)r * G * d,
                       lse + (size_t)r * G, z, o);
        }
        free(keys);
        free(z);
        free(o);
    }
}

/* Gradient of stage 4 (Appendix Alg. 2, or Eq. 1 when idx == NULL) with respect to Q, K and V for a given
 * selection; the selection itself (stages 1-3) is piecewise constant and carries no gradient (Sec. 3.3: the
 * compressed scores only pick blocks).  Written from the definition O = softmax(z) V, z_a = scale <q, k_a>:
 *   p = softmax(z),  dp_a = <dO, v_a>,  D = sum_a p_a dp_a,  dz_a = p_a (dp_a - D),
 *   dq = scale sum_a dz_a k_a,   dk_a += scale dz_a q,   dv_a += p_a dO
 * per query row and head, everything in double.  dO [nr][G][d]; dQ [nr][G][d]; dK, dV [n][d] are ACCUMULATED
 * into (the caller zeroes them), so that several row subsets can be summed. */
void oracle_attn_bwd(const float *Q, const int32_t *pos, int nr, int G, int d, const float *K, const float *V,
                     int n, int B, const int32_t *idx, int topk_total, double scale, const float *dO,
                     double *dQ, double *dK, double *dV) {
    int cap = idx ? topk_total * B : (n > 0 ? n : 1);
    int *keys = (int *)malloc(sizeof(int) * (size_t)cap);
    double *p = (double *)malloc(sizeof(double) * (size_t)cap);
    for (int r = 0; r < nr; ++r) {
        int t = pos[r];
        int nk = 0;
        if (idx) {
            for (int s = 0; s < topk_total; ++s) {
                int j = idx[(size_t)r * topk_total + s];
                if (j < 0) continue;
                for (int u = j * B; u < (j + 1) * B && u <= t && u < n; ++u) keys[nk++] = u;
            }
        } else {
            for (int u = 0; u <= t && u < n; ++u) keys[nk++] = u;
        }
        for (int g = 0; g < G; ++g) {
            const float *q = Q + ((size_t)r * G + g) * d;
            const float *go = dO + ((size_t)r * G + g) * d;
            double *gq = dQ + ((size_t)r * G + g) * d;
            double zmax = -INFINITY;
            for (int a = 0; a < nk; ++a) {
                const float *kr = K + (size_t)keys[a] * d;
                double dot = 0.0;
                for (int c = 0; c < d; ++c) dot += (double)q[c] * (double)kr[c];
                p[a] = scale * dot;
                if (p[a] > zmax) zmax = p[a];
            }
            double den = 0.0;
            for (int a = 0; a < nk; ++a) {
                p[a] = exp(p[a] - zmax);
                den += p[a];
            }
            double D = 0.0;
            for (int a = 0; a < nk; ++a) {
                p[a] /= den;
                const float *vr = V + (size_t)keys[a] * d;
                double dp = 0.0;
                for (int c = 0; c < d; ++c) dp += (double)go[c] * (double)vr[c];
                D += p[a] * dp;
            }
            for (int c = 0; c < d; ++c) gq[c] = 0.0;
            for (int a = 0; a < nk; ++a) {
                const float *kr = K + (size_t)keys[a] * d;
                const float *vr = V + (size_t)keys[a] * d;
                double dp = 0.0;
                for (int c = 0; c < d; ++c) dp += (double)go[c] * (double)vr[c];
                const double dz = p[a] * (dp - D);
                double *gk = dK + (size_t)keys[a] * d, *gv = dV + (size_t)keys[a] * d;
                for (int c = 0; c < d; ++c) {
                    gq[c] += scale * dz * (double)kr[c];
                    gk[c] += scale * dz * (double)q[c];
                    gv[c] += p[a] * (double)go[c];
                }
            }
        }
    }
    free(keys);
    free(p);
}

