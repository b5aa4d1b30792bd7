/* CPU oracle for the NAtS-L hybrid attention operator, C version
 * (TEST INFRASTRUCTURE ONLY -- the product path never links or loads this).
 *
 * Same definitions as the numpy oracle beside it, written token by token in
 * fp64 so that full-size workloads finish in seconds; OpenMP runs the
 * independent (batch, head) pairs side by side.  Shares no code with the HIP
 * kernels.
 *
 *   linear branch : Gated DeltaNet recurrence, Section 4.3 Eq. 19, written only
 *                   for linear tokens (Eq. 14), decay at every token (Eq. 20),
 *                   read by every query o_t = S_t q_t (Eq. 5 / Eq. 10)
 *   softmax branch: Eq. 11 under the column mask of Eq. 12
 *   merge         : sum (Section 4.1) or Eq. 21 with given weights
 *
 * Inputs are float32 (bf16 workloads hand in bf16-representable floats), all
 * arithmetic is double, outputs are double.
 *
 * Parity pins: tests/test_oracle_pins.py runs the same pins against this
 * library as against the numpy oracle.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Variants of the linear branch, set before a call and read by every function below (the defaults are the
 * method as stated):
 *   g_linear_op = 1        : the linear operation is the gated linear attention of Mamba2,
 *                            S_t = alpha_t S_{t-1} + beta_t v_t k_t^T (no delta correction), the second linear
 *                            operation of the appendix "Mixture of SoftmaxAttention and Mamba2 architecture"
 *   g_freeze_on_softmax = 1: no decay where the state is not written (the ablation without linear-attention
 *                            decay, Section 5 "Ablation Study" (ii), i.e. Eq. 20 switched off) */
static int g_linear_op = 0, g_freeze_on_softmax = 0;
void nats_oracle_set_variant(int linear_op, int freeze_on_softmax) {
    g_linear_op = linear_op;
    g_freeze_on_softmax = freeze_on_softmax;
}

int nats_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One (batch, head).  S is d x d row-major [d_v][d_k], updated in place. */
static void head_forward(int L, int d, const float *q, const float *k, const float *v,
                         const float *alpha, const float *beta, const uint8_t *mask,
                         double scale, double la_scale, int mode, const float *w_nla,
                         const float *w_la, double eps, double *S, double *O, double *O_la,
                         double *O_nla, double *lse, int32_t *cnt, int32_t *idx, int32_t *n_s_out) {
    double *pred = (double *)malloc(sizeof(double) * d);
    double *ola = (double *)malloc(sizeof(double) * d);
    double *onla = (double *)malloc(sizeof(double) * d);
    double *score = (double *)malloc(sizeof(double) * (L > 0 ? L : 1));
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (L > 0 ? L : 1));
    int n_s = 0;
    for (int t = 0; t < L; ++t) {
        const float *qt = q + (size_t)t * d, *kt = k + (size_t)t * d, *vt = v + (size_t)t * d;
        /* ---- linear branch ---- */
        double a = (mask[t] != 0 && g_freeze_on_softmax) ? 1.0 : alpha[t];
        for (int i = 0; i < d * d; ++i) S[i] *= a;                 /* Eq. 20: decay always */
        if (mask[t] == 0) {                                        /* Eq. 14: write linear tokens only */
            double b = beta[t];
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                if (g_linear_op == 0)
                    for (int c = 0; c < d; ++c) acc += S[r * d + c] * (double)kt[c];
                pred[r] = acc;
            }
            for (int r = 0; r < d; ++r) {                          /* Eq. 19 expanded */
                double delta = b * ((double)vt[r] - pred[r]);
                for (int c = 0; c < d; ++c) S[r * d + c] += delta * (double)kt[c];
            }
        } else {
            pos[n_s] = t;                                          /* softmax column (Eq. 12) */
            n_s += 1;
        }
        if (cnt) cnt[t] = n_s;
        for (int r = 0; r < d; ++r) {                              /* Eq. 5 */
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += S[r * d + c] * (double)qt[c];
            ola[r] = la_scale * acc;
        }
        /* ---- softmax branch over the softmax columns j <= t ---- */
        double row_lse = -INFINITY;
        for (int r = 0; r < d; ++r) onla[r] = 0.0;
        if (n_s > 0) {
            double smax = -INFINITY;
            for (int c = 0; c < n_s; ++c) {
                const float *kj = k + (size_t)pos[c] * d;
                double acc = 0.0;
                for (int i = 0; i < d; ++i) acc += (double)qt[i] * (double)kj[i];
                score[c] = scale * acc;
                if (score[c] > smax) smax = score[c];
            }
            double z = 0.0;
            for (int c = 0; c < n_s; ++c) {
                score[c] = exp(score[c] - smax);
                z += score[c];
            }
            for (int c = 0; c < n_s; ++c) {
                const float *vj = v + (size_t)pos[c] * d;
                double p = score[c] / z;
                for (int r = 0; r < d; ++r) onla[r] += p * (double)vj[r];
            }
            row_lse = smax + log(z);
        }
        /* ---- merge ---- */
        double *o = O + (size_t)t * d;
        if (mode == 0) {
            for (int r = 0; r < d; ++r) o[r] = ola[r] + onla[r];
        } else if (mode == 2) {                                   /* one normalisation of the weighted sum */
            double wn = w_nla ? (double)w_nla[t] : 1.0, wl = w_la ? (double)w_la[t] : 1.0, ms = 0.0;
            for (int r = 0; r < d; ++r) { o[r] = wn * onla[r] + wl * ola[r]; ms += o[r] * o[r]; }
            double inv = 1.0 / sqrt(ms / d + eps);
            for (int r = 0; r < d; ++r) o[r] *= inv;
        } else {
            double ms_la = 0.0, ms_nla = 0.0;
            for (int r = 0; r < d; ++r) { ms_la += ola[r] * ola[r]; ms_nla += onla[r] * onla[r]; }
            double inv_la = 1.0 / sqrt(ms_la / d + eps), inv_nla = 1.0 / sqrt(ms_nla / d + eps);
            double wn = w_nla ? (double)w_nla[t] : 0.5, wl = w_la ? (double)w_la[t] : 0.5;
            for (int r = 0; r < d; ++r) o[r] = wn * onla[r] * inv_nla + wl * ola[r] * inv_la;
        }
        if (O_la) memcpy(O_la + (size_t)t * d, ola, sizeof(double) * d);
        if (O_nla) memcpy(O_nla + (size_t)t * d, onla, sizeof(double) * d);
        if (lse) lse[t] = row_lse;
    }
    if (idx) for (int c = 0; c < n_s; ++c) idx[c] = pos[c];
    if (n_s_out) *n_s_out = n_s;
    free(pred); free(ola); free(onla); free(score); free(pos);
}

/* Q,K,V [BH,L,d] float; alpha,beta [BH,L] float; mask [BH,L] u8;
 * S0 [BH,d,d] double or NULL (zero); outputs double / int32, any of
 * O_la,O_nla,lse,S_final,cnt,idx,n_s may be NULL.  idx is [BH,L].
 * Returns 0, or -1 on a bad argument. */
int nats_oracle_fwd(int BH, int L, int d, const float *Q, const float *K, const float *V,
                    const float *alpha, const float *beta, const uint8_t *mask, double scale,
                    double la_scale, int mode, const float *w_nla, const float *w_la, double eps,
                    const double *S0, double *O, double *O_la, double *O_nla, double *lse,
                    double *S_final, int32_t *cnt, int32_t *idx, int32_t *n_s) {
    if (!Q || !K || !V || !alpha || !beta || !mask || !O || BH < 0 || L < 0 || d <= 0) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < BH; ++u) {
        size_t ld = (size_t)L * d, off = (size_t)u * ld, offl = (size_t)u * L;
        double *S = (double *)malloc(sizeof(double) * d * d);
        if (S0) memcpy(S, S0 + (size_t)u * d * d, sizeof(double) * d * d);
        else memset(S, 0, sizeof(double) * d * d);
        head_forward(L, d, Q + off, K + off, V + off, alpha + offl, beta + offl, mask + offl, scale,
                     la_scale, mode, w_nla ? w_nla + offl : NULL, w_la ? w_la + offl : NULL, eps, S,
                     O + off, O_la ? O_la + off : NULL, O_nla ? O_nla + off : NULL,
                     lse ? lse + offl : NULL, cnt ? cnt + offl : NULL, idx ? idx + offl : NULL,
                     n_s ? n_s + u : NULL);
        if (S_final) memcpy(S_final + (size_t)u * d * d, S, sizeof(double) * d * d);
        free(S);
    }
    return 0;
}

/* One decode token for BH independent (batch, head) pairs (Section 4.1, per-token
 * generation).  state [BH,d,d] double in place; caches [BH,cap,d] float in place
 * (they only ever hold input values verbatim);
 * cache_len [BH] in place; q,k,v [BH,d] float; alpha,beta [BH] float; mask [BH];
 * o [BH,d] double; overflow [BH] set to 1 where a softmax token found the cache full. */
int nats_oracle_decode(int BH, int d, int cap, double *state, float *k_cache, float *v_cache,
                       int32_t *cache_len, const float *q, const float *k, const float *v,
                       const float *alpha, const float *beta, const uint8_t *mask, double scale,
                       double la_scale, int mode, const float *w_nla, const float *w_la, double eps,
                       double *o, int32_t *overflow) {
    if (!state || !k_cache || !v_cache || !cache_len || !q || !k || !v || !o) return -1;
#pragma omp parallel for schedule(static)
    for (int u = 0; u < BH; ++u) {
        double *S = state + (size_t)u * d * d;
        float *kc = k_cache + (size_t)u * cap * d, *vc = v_cache + (size_t)u * cap * d;
        const float *qt = q + (size_t)u * d, *kt = k + (size_t)u * d, *vt = v + (size_t)u * d;
        double a = (mask[u] != 0 && g_freeze_on_softmax) ? 1.0 : alpha[u];
        for (int i = 0; i < d * d; ++i) S[i] *= a;
        if (overflow) overflow[u] = 0;
        if (mask[u] == 0) {
            double b = beta[u];
            double *pred = (double *)malloc(sizeof(double) * d);
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                if (g_linear_op == 0)
                    for (int c = 0; c < d; ++c) acc += S[r * d + c] * (double)kt[c];
                pred[r] = acc;
            }
            for (int r = 0; r < d; ++r) {
                double delta = b * ((double)vt[r] - pred[r]);
                for (int c = 0; c < d; ++c) S[r * d + c] += delta * (double)kt[c];
            }
            free(pred);
        } else if (cache_len[u] < cap) {
            int n = cache_len[u];
            for (int i = 0; i < d; ++i) { kc[(size_t)n * d + i] = kt[i]; vc[(size_t)n * d + i] = vt[i]; }
            cache_len[u] = n + 1;
        } else if (overflow) {
            overflow[u] = 1;
        }
        double *ola = (double *)malloc(sizeof(double) * d);
        double *onla = (double *)calloc(d, sizeof(double));
        for (int r = 0; r < d; ++r) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += S[r * d + c] * (double)qt[c];
            ola[r] = la_scale * acc;
        }
        int n = cache_len[u];
        if (n > 0) {
            double *score = (double *)malloc(sizeof(double) * n);
            double smax = -INFINITY, z = 0.0;
            for (int c = 0; c < n; ++c) {
                double acc = 0.0;
                for (int i = 0; i < d; ++i) acc += (double)qt[i] * (double)kc[(size_t)c * d + i];
                score[c] = scale * acc;
                if (score[c] > smax) smax = score[c];
            }
            for (int c = 0; c < n; ++c) { score[c] = exp(score[c] - smax); z += score[c]; }
            for (int c = 0; c < n; ++c) {
                double p = score[c] / z;
                for (int r = 0; r < d; ++r) onla[r] += p * (double)vc[(size_t)c * d + r];
            }
            free(score);
        }
        double *out = o + (size_t)u * d;
        if (mode == 0) {
            for (int r = 0; r < d; ++r) out[r] = ola[r] + onla[r];
        } else if (mode == 2) {
            double wn = w_nla ? (double)w_nla[u] : 1.0, wl = w_la ? (double)w_la[u] : 1.0, ms = 0.0;
            for (int r = 0; r < d; ++r) { out[r] = wn * onla[r] + wl * ola[r]; ms += out[r] * out[r]; }
            double inv = 1.0 / sqrt(ms / d + eps);
            for (int r = 0; r < d; ++r) out[r] *= inv;
        } else {
            double ms_la = 0.0, ms_nla = 0.0;
            for (int r = 0; r < d; ++r) { ms_la += ola[r] * ola[r]; ms_nla += onla[r] * onla[r]; }
            double inv_la = 1.0 / sqrt(ms_la / d + eps), inv_nla = 1.0 / sqrt(ms_nla / d + eps);
            double wn = w_nla ? (double)w_nla[u] : 0.5, wl = w_la ? (double)w_la[u] : 0.5;
            for (int r = 0; r < d; ++r) out[r] = wn * onla[r] * inv_nla + wl * ola[r] * inv_la;
        }
        free(ola); free(onla);
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Chunk-level routing (Section 4.1 as stated: one decision per chunk of C tokens,
 * taken after the chunk has been seen).  Both operations compute the intra-chunk part
 * of every chunk; afterwards the operation that was not chosen is rolled back:
 *   linear branch : Eq. 19 on every token of the chunk from the chunk-start state; after a
 *                   softmax chunk the state is reset to (chunk decay) x (chunk-start state)
 *                   (writes dropped, Eq. 14; decay kept, Eq. 20)
 *   softmax branch: keys = tokens of earlier softmax chunks (Eq. 12 per chunk) plus the
 *                   tokens j <= t of the query's own chunk
 * mask_c is [BH, L/C]; everything else as in nats_oracle_fwd (cnt, idx, n_s: compaction of
 * the tokens of softmax chunks). */
static void head_forward_chunk(int L, int d, int C, const float *q, const float *k, const float *v,
                               const float *alpha, const float *beta, const uint8_t *mask_c,
                               double scale, double la_scale, int mode, const float *w_nla,
                               const float *w_la, double eps, double *S, double *O, double *O_la,
                               double *O_nla, double *lse, int32_t *cnt, int32_t *idx, int32_t *n_s_out) {
    double *pred = (double *)malloc(sizeof(double) * d);
    double *ola = (double *)malloc(sizeof(double) * d);
    double *onla = (double *)malloc(sizeof(double) * d);
    double *score = (double *)malloc(sizeof(double) * (L > 0 ? L : 1));
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (L > 0 ? L : 1));   /* visible key positions */
    double *S_start = (double *)malloc(sizeof(double) * d * d);
    int n_s = 0;                                   /* tokens of earlier softmax chunks */
    for (int c0 = 0; c0 < L; c0 += C) {
        const int soft = mask_c[c0 / C] != 0;
        memcpy(S_start, S, sizeof(double) * d * d);
        double decay = 1.0;
        for (int t = c0; t < c0 + C; ++t) {
            const float *qt = q + (size_t)t * d, *kt = k + (size_t)t * d, *vt = v + (size_t)t * d;
            double a = alpha[t], b = beta[t];
            decay *= a;
            for (int i = 0; i < d * d; ++i) S[i] *= a;
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                if (g_linear_op == 0)
                    for (int j = 0; j < d; ++j) acc += S[r * d + j] * (double)kt[j];
                pred[r] = acc;
            }
            for (int r = 0; r < d; ++r) {                           /* Eq. 19, every token of the chunk */
                double delta = b * ((double)vt[r] - pred[r]);
                for (int j = 0; j < d; ++j) S[r * d + j] += delta * (double)kt[j];
            }
            for (int r = 0; r < d; ++r) {
                double acc = 0.0;
                for (int j = 0; j < d; ++j) acc += S[r * d + j] * (double)qt[j];
                ola[r] = la_scale * acc;
            }
            /* visible keys: pos[0..n_s) from earlier softmax chunks, then c0..t of the own chunk */
            const int n_vis = n_s + (t - c0 + 1);
            double smax = -INFINITY, z = 0.0;
            for (int cc = 0; cc < n_vis; ++cc) {
                const int j = cc < n_s ? pos[cc] : c0 + (cc - n_s);
                const float *kj = k + (size_t)j * d;
                double acc = 0.0;
                for (int i = 0; i < d; ++i) acc += (double)qt[i] * (double)kj[i];
                score[cc] = scale * acc;
                if (score[cc] > smax) smax = score[cc];
            }
            for (int cc = 0; cc < n_vis; ++cc) { score[cc] = exp(score[cc] - smax); z += score[cc]; }
            for (int r = 0; r < d; ++r) onla[r] = 0.0;
            for (int cc = 0; cc < n_vis; ++cc) {
                const int j = cc < n_s ? pos[cc] : c0 + (cc - n_s);
                const float *vj = v + (size_t)j * d;
                double p = score[cc] / z;
                for (int r = 0; r < d; ++r) onla[r] += p * (double)vj[r];
            }
            double *o = O + (size_t)t * d;
            if (mode == 0) {
                for (int r = 0; r < d; ++r) o[r] = ola[r] + onla[r];
            } else if (mode == 2) {
                double wn = w_nla ? (double)w_nla[t] : 1.0, wl = w_la ? (double)w_la[t] : 1.0, ms = 0.0;
                for (int r = 0; r < d; ++r) { o[r] = wn * onla[r] + wl * ola[r]; ms += o[r] * o[r]; }
                double inv = 1.0 / sqrt(ms / d + eps);
                for (int r = 0; r < d; ++r) o[r] *= inv;
            } else {
                double ms_la = 0.0, ms_nla = 0.0;
                for (int r = 0; r < d; ++r) { ms_la += ola[r] * ola[r]; ms_nla += onla[r] * onla[r]; }
                double inv_la = 1.0 / sqrt(ms_la / d + eps), inv_nla = 1.0 / sqrt(ms_nla / d + eps);
                double wn = w_nla ? (double)w_nla[t] : 0.5, wl = w_la ? (double)w_la[t] : 0.5;
                for (int r = 0; r < d; ++r) o[r] = wn * onla[r] * inv_nla + wl * ola[r] * inv_la;
            }
            if (O_la) memcpy(O_la + (size_t)t * d, ola, sizeof(double) * d);
            if (O_nla) memcpy(O_nla + (size_t)t * d, onla, sizeof(double) * d);
            if (lse) lse[t] = smax + log(z);
            if (cnt) cnt[t] = n_s + (soft ? (t - c0 + 1) : 0);
        }
        if (soft) {
            if (g_freeze_on_softmax) decay = 1.0;
            for (int i = 0; i < d * d; ++i) S[i] = decay * S_start[i];   /* writes rolled back */
            for (int t = c0; t < c0 + C; ++t) pos[n_s++] = t;
        }
    }
    if (idx) for (int c = 0; c < n_s; ++c) idx[c] = pos[c];
    if (n_s_out) *n_s_out = n_s;
    free(pred); free(ola); free(onla); free(score); free(pos); free(S_start);
}

int nats_oracle_fwd_chunk(int BH, int L, int d, int C, const float *Q, const float *K, const float *V,
                          const float *alpha, const float *beta, const uint8_t *mask_c, double scale,
                          double la_scale, int mode, const float *w_nla, const float *w_la, double eps,
                          const double *S0, double *O, double *O_la, double *O_nla, double *lse,
                          double *S_final, int32_t *cnt, int32_t *idx, int32_t *n_s) {
    if (!Q || !K || !V || !alpha || !beta || !mask_c || !O || BH < 0 || L < 0 || d <= 0 || C <= 0 || L % C) return -1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < BH; ++u) {
        size_t ld = (size_t)L * d, off = (size_t)u * ld, offl = (size_t)u * L;
        double *S = (double *)malloc(sizeof(double) * d * d);
        if (S0) memcpy(S, S0 + (size_t)u * d * d, sizeof(double) * d * d);
        else memset(S, 0, sizeof(double) * d * d);
        head_forward_chunk(L, d, C, Q + off, K + off, V + off, alpha + offl, beta + offl,
                           mask_c + (size_t)u * (L / C), scale, la_scale, mode, w_nla ? w_nla + offl : NULL,
                           w_la ? w_la + offl : NULL, eps, S, O + off, O_la ? O_la + off : NULL,
                           O_nla ? O_nla + off : NULL, lse ? lse + offl : NULL, cnt ? cnt + offl : NULL,
                           idx ? idx + offl : NULL, n_s ? n_s + u : NULL);
        if (S_final) memcpy(S_final + (size_t)u * d * d, S, sizeof(double) * d * d);
        free(S);
    }
    return 0;
}
