/*
 * CPU checker ("oracle") for the selective-rollout decode path.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product library may include, link
 * or call this file; it exists so that the GPU kernels can be compared against
 * a plain, slow, obviously-correct evaluation of the same quantities.
 *
 * Everything is written out directly from its definition:
 *   - Levenshtein distance: full (m+1) x (n+1) table, unit costs.
 *   - Gate: the paper's Section 3.2 signal d_K (mean over the C(G,2) pairs of
 *     the prefix edit distance divided by the longer length) and the decision
 *     of Eq. 2, cut iff d_K < d_L, evaluated in integers.
 *   - The other in-group signals of Appendix B (action-bigram Jaccard, unique
 *     prefix / action / observation counts, action entropy, termination
 *     fraction), d_K for members that finished early (each pair divided by
 *     the longer of its two prefix lengths) and the two-clause gate of
 *     Appendix E (Eq. 3), decided in exact integer arithmetic.
 *   - Advantage: Eq. 1 (population standard deviation); the teacher-forced
 *     log-likelihood of Appendix C.2 (log-softmax at action-token positions)
 *     and the policy-gradient loss built from the two.
 *   - Decoder: pre-norm transformer decoder (RMSNorm, biased QKV projection,
 *     rotate-half RoPE, grouped-query causal attention, SwiGLU FFN, untied LM
 *     head), one token at a time over a flat per-sequence KV list.  No paging,
 *     no sharing, no blocking, no fusion.
 *
 * Floating point type: `real`, double unless SRO_REAL is defined otherwise
 * (a second build with -DSRO_REAL=float exists to measure the precision scale).
 * Weights arrive as bf16 bit patterns and are widened exactly.
 */
#include <limits.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef SRO_REAL
#define SRO_REAL double
#endif
typedef SRO_REAL real;

int sro_real_bytes(void) { return (int)sizeof(real); }

/* ------------------------------------------------------------------------- */
/* Levenshtein distance (textbook full table; insert/delete/substitute cost 1) */
/* ------------------------------------------------------------------------- */
int sro_lev(const int32_t *a, int m, const int32_t *b, int n) {
    int *D = (int *)malloc((size_t)(m + 1) * (size_t)(n + 1) * sizeof(int));
    const int W = n + 1;
    for (int i = 0; i <= m; ++i) D[i * W] = i;
    for (int j = 0; j <= n; ++j) D[j] = j;
    for (int i = 1; i <= m; ++i) {
        for (int j = 1; j <= n; ++j) {
            int del = D[(i - 1) * W + j] + 1;
            int ins = D[i * W + (j - 1)] + 1;
            int sub = D[(i - 1) * W + (j - 1)] + (a[i - 1] != b[j - 1] ? 1 : 0);
            int best = del < ins ? del : ins;
            D[i * W + j] = best < sub ? best : sub;
        }
    }
    int r = D[m * W + n];
    free(D);
    return r;
}

/*
 * S_K = sum over pairs i<j of lev(a_i[0:K], a_j[0:K]) for one group whose G
 * members all hold at least K actions (Section 3.2; equal lengths, so every
 * pair is normalised by the same K and d_K = S_K / (C(G,2) * K)).
 * actions is [G][stride].
 */
int64_t sro_pair_sum(const int32_t *actions, int G, int stride, int K) {
    int64_t s = 0;
    for (int i = 0; i < G; ++i)
        for (int j = i + 1; j < G; ++j)
            s += sro_lev(actions + (size_t)i * stride, K, actions + (size_t)j * stride, K);
    return s;
}

/*
 * Integer form of Eq. 2.  d_L is resolved to a rational num/1e6 with
 * num = round(d_L * 1e6).  With P = C(G,2):
 *   d_K < d_L  <=>  S_K / (P*K) < num/1e6  <=>  S_K * 1e6 < num * P * K
 *             <=>  S_K < ceil(num*P*K / 1e6)          (S_K integer)
 * Returns that ceiling; the group is cut iff S_K < return value.
 */
int64_t sro_gate_bound(double d_L, int G, int K) {
    const int64_t den = 1000000;
    int64_t num = (int64_t)llround(d_L * 1e6);
    int64_t P = (int64_t)G * (G - 1) / 2;
    int64_t rhs = num * P * (int64_t)K;
    return (rhs + den - 1) / den;
}

/* d_K as a floating-point number, for reporting only. */
double sro_mean_prefix_distance(const int32_t *actions, int G, int stride, int K) {
    double P = 0.5 * G * (G - 1);
    return (double)sro_pair_sum(actions, G, stride, K) / (P * K);
}

/*
 * Gate over many groups and several prefix lengths.
 * actions [n_groups][G][stride]; sums / cut are [n_lens][n_groups].
 */
void sro_gate_batch(const int32_t *actions, int n_groups, int G, int stride,
                    const int32_t *lens, int n_lens, double d_L,
                    int32_t *sums, uint8_t *cut) {
    for (int li = 0; li < n_lens; ++li) {
        const int K = lens[li];
        const int64_t bound = sro_gate_bound(d_L, G, K);
#pragma omp parallel for schedule(static)
        for (int g = 0; g < n_groups; ++g) {
            int64_t s = sro_pair_sum(actions + (size_t)g * G * stride, G, stride, K);
            sums[(size_t)li * n_groups + g] = (int32_t)s;
            cut[(size_t)li * n_groups + g] = (uint8_t)(s < bound);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* In-group divergence signals at step K (Appendix B) and the two-clause gate  */
/* (Appendix E, Eq. 3), for groups whose members may have finished early.      */
/* ------------------------------------------------------------------------- */
/*
 * Member i finished after end_step[i] environment steps (a large value while it
 * is still running), so at step K it contributes the prefix a_i[0 : len_i] with
 * len_i = min(K, end_step[i]).  A pair's edit distance is divided by the longer
 * of its two prefix lengths (Section 3.2); a pair of two empty prefixes counts 0.
 *
 * The sum of the pair terms is also kept exactly, as an integer multiple of
 * 1 / SRO_LCM32 where SRO_LCM32 = lcm(1..32): lev * (SRO_LCM32 / longer) summed
 * over pairs.  Eq. 2 is then decided without rounding:
 *   d_K < d_L  <=>  lev_scaled / (P * LCM) < num / 1e6  <=>  lev_scaled * 1e6 < num * P * LCM.
 */
#define SRO_LCM32 144403552893600LL

typedef struct {
    double d_K;               /* mean over pairs of lev / longer length                              */
    int64_t lev_scaled;       /* sum over pairs of lev * (SRO_LCM32 / longer length)                 */
    double bigram_jaccard;    /* mean over pairs of 1 - |A n B| / |A u B|, A, B = sets of action bigrams */
    double action_entropy;    /* Shannon entropy (nats) of the step-K action over members at step K   */
    int32_t unique_prefix;    /* distinct prefixes among the G members                                */
    int32_t n_at_step;        /* members whose prefix reaches step K (len_i == K)                     */
    int32_t unique_action;    /* distinct a_{i,K} among them                                          */
    int32_t unique_obs;       /* distinct o_{i,K} among them                                          */
    int32_t n_done;           /* members that had finished by step K (end_step <= K)                  */
    int32_t lev_sum;          /* plain sum over pairs of the edit distances                           */
    uint8_t cut_d;            /* Eq. 2: d_K < d_L                                                     */
    uint8_t cut_or;           /* Eq. 3: d_K < d_L or tau_K >= tau_H, tau_K = n_done / G               */
} sro_signals_t;

static int distinct_bigrams(const int32_t *a, int len, int32_t (*out)[2]) {
    int n = 0;
    for (int t = 0; t + 1 < len; ++t) {
        int seen = 0;
        for (int u = 0; u < n; ++u)
            if (out[u][0] == a[t] && out[u][1] == a[t + 1]) seen = 1;
        if (!seen) { out[n][0] = a[t]; out[n][1] = a[t + 1]; ++n; }
    }
    return n;
}

/* actions, obs: [G][stride] (obs may be NULL); end_step: [G] or NULL (nobody has finished). K <= 32, K <= stride. */
void sro_signals(const int32_t *actions, const int32_t *obs, const int32_t *end_step, int G, int stride, int K,
                 double d_L, double tau_H, sro_signals_t *out) {
    int len[64];
    int n_done = 0;
    for (int i = 0; i < G; ++i) {
        const int e = end_step ? end_step[i] : INT32_MAX;
        len[i] = e < K ? e : K;
        if (e <= K) ++n_done;
    }
    const int64_t P = (int64_t)G * (G - 1) / 2;

    /* mean pairwise prefix edit distance, and the action-bigram Jaccard distance */
    double dsum = 0.0, jsum = 0.0;
    int64_t scaled = 0;
    int32_t plain = 0;
    for (int i = 0; i < G; ++i)
        for (int j = i + 1; j < G; ++j) {
            const int32_t *a = actions + (size_t)i * stride, *b = actions + (size_t)j * stride;
            const int longer = len[i] > len[j] ? len[i] : len[j];
            if (longer > 0) {
                const int d = sro_lev(a, len[i], b, len[j]);
                plain += d;
                dsum += (double)d / (double)longer;
                scaled += (int64_t)d * (SRO_LCM32 / longer);
            }
            int32_t A[32][2], B[32][2];
            const int na = distinct_bigrams(a, len[i], A), nb = distinct_bigrams(b, len[j], B);
            int inter = 0;
            for (int u = 0; u < na; ++u)
                for (int v = 0; v < nb; ++v)
                    if (A[u][0] == B[v][0] && A[u][1] == B[v][1]) ++inter;
            const int uni = na + nb - inter;
            jsum += uni > 0 ? 1.0 - (double)inter / (double)uni : 0.0;   /* two empty sets: identical */
        }
    out->d_K = dsum / (double)P;
    out->lev_scaled = scaled;
    out->lev_sum = plain;
    out->bigram_jaccard = jsum / (double)P;

    /* distinct prefixes */
    int uniq = 0;
    for (int i = 0; i < G; ++i) {
        int dup = 0;
        for (int j = 0; j < i; ++j)
            if (len[j] == len[i] && memcmp(actions + (size_t)i * stride, actions + (size_t)j * stride,
                                           (size_t)len[i] * sizeof(int32_t)) == 0)
                dup = 1;
        if (!dup) ++uniq;
    }
    out->unique_prefix = uniq;

    /* the single step-K action / observation, over the members that reach step K */
    int n_at = 0, ua = 0, uo = 0;
    double H = 0.0;
    for (int i = 0; i < G; ++i) n_at += len[i] == K;
    for (int i = 0; i < G; ++i) {
        if (len[i] != K) continue;
        const int32_t ai = actions[(size_t)i * stride + K - 1];
        int first_a = 1, first_o = 1, count = 0;
        for (int j = 0; j < G; ++j) {
            if (len[j] != K) continue;
            const int same_a = actions[(size_t)j * stride + K - 1] == ai;
            if (same_a) ++count;
            if (j < i && same_a) first_a = 0;
            if (obs && j < i && obs[(size_t)j * stride + K - 1] == obs[(size_t)i * stride + K - 1]) first_o = 0;
        }
        if (first_a) {
            ++ua;
            const double p = (double)count / (double)n_at;
            H -= p * log(p);
        }
        if (obs && first_o) ++uo;
    }
    out->n_at_step = n_at;
    out->unique_action = ua;
    out->unique_obs = obs ? uo : 0;
    out->action_entropy = H;
    out->n_done = n_done;

    const int64_t num_d = (int64_t)llround(d_L * 1e6), num_t = (int64_t)llround(tau_H * 1e6);
    out->cut_d = (uint8_t)((__int128)scaled * 1000000 < (__int128)num_d * P * SRO_LCM32);
    out->cut_or = (uint8_t)(out->cut_d || (int64_t)n_done * 1000000 >= num_t * G);
}

/* actions/obs [n_groups][G][stride], end_step [n_groups][G]; out [n_lens][n_groups] */
void sro_signals_batch(const int32_t *actions, const int32_t *obs, const int32_t *end_step, int n_groups, int G,
                       int stride, const int32_t *lens, int n_lens, double d_L, double tau_H, sro_signals_t *out) {
    for (int li = 0; li < n_lens; ++li) {
#pragma omp parallel for schedule(static)
        for (int g = 0; g < n_groups; ++g)
            sro_signals(actions + (size_t)g * G * stride, obs ? obs + (size_t)g * G * stride : NULL,
                        end_step ? end_step + (size_t)g * G : NULL, G, stride, lens[li], d_L, tau_H,
                        out + (size_t)li * n_groups + g);
    }
}

int64_t sro_lcm32(void) { return SRO_LCM32; }

/* ------------------------------------------------------------------------- */
/* Group-relative advantage, Eq. 1                                            */
/* ------------------------------------------------------------------------- */
void sro_advantage(const double *r, int G, double eps, double *A) {
    int all_equal = 1;
    for (int i = 1; i < G; ++i)
        if (r[i] != r[0]) all_equal = 0;
    if (all_equal) {            /* sigma_r = 0: every advantage is exactly zero (Section 2.1) */
        for (int i = 0; i < G; ++i) A[i] = 0.0;
        return;
    }
    double mean = 0.0;
    for (int i = 0; i < G; ++i) mean += r[i];
    mean /= G;
    double var = 0.0;
    for (int i = 0; i < G; ++i) var += (r[i] - mean) * (r[i] - mean);
    double sigma = sqrt(var / G);
    for (int i = 0; i < G; ++i) A[i] = (r[i] - mean) / (sigma + eps);
}

/* ------------------------------------------------------------------------- */
/* Decoder                                                                    */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, qkv_bias;
    double rms_eps, rope_theta;
} sro_shape;

typedef struct {
    /* bf16 bit patterns, matrices row-major [out_features][in_features] */
    const uint16_t *wq, *wk, *wv, *wo, *wg, *wu, *wd, *bq, *bk, *bv, *norm1, *norm2;
} sro_layer;

typedef struct {
    sro_shape s;
    const uint16_t *embed, *lm_head, *final_norm;
    sro_layer *layers;
} sro_model;

typedef struct {
    int len, cap;
    real *k; /* [n_layers][cap][n_kv_heads*head_dim] */
    real *v;
} sro_seq;

/*
 * Optional "bf16 contract" mode (off by default): activations are rounded to bf16 (nearest even)
 * at exactly the points where a bf16 tensor-core implementation must round them -- the inputs of
 * every projection, the stored keys and values, the rotated queries and the softmax probabilities
 * fed to the value product -- and nowhere else.  It separates the error that is inherent to bf16
 * operands from implementation error: an implementation should agree with this mode far more
 * closely than with the exact evaluation.
 */
static int g_contract = 0;
void sro_set_bf16_contract(int on) { g_contract = on; }

/*
 * The rounding itself, exported so that tests can pin it: the value is first rounded to
 * single precision (the accumulators whose contents become bf16 operands are single precision),
 * then to the nearest bf16 (8 significant bits), ties to the even significand; a carry may
 * move into the exponent.  Finite inputs only.
 */
double sro_bf16_round(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

static inline real rb(real x) { return g_contract ? (real)sro_bf16_round((double)x) : x; }

static inline real bf16_to_real(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (real)f;
}

sro_model *sro_model_new(const sro_shape *s, const uint16_t *embed, const uint16_t *lm_head,
                         const uint16_t *final_norm) {
    sro_model *m = (sro_model *)calloc(1, sizeof(sro_model));
    m->s = *s;
    m->embed = embed;
    m->lm_head = lm_head;
    m->final_norm = final_norm;
    m->layers = (sro_layer *)calloc((size_t)s->n_layers, sizeof(sro_layer));
    return m;
}

void sro_model_set_layer(sro_model *m, int l, const uint16_t *wq, const uint16_t *wk,
                         const uint16_t *wv, const uint16_t *wo, const uint16_t *wg,
                         const uint16_t *wu, const uint16_t *wd, const uint16_t *bq,
                         const uint16_t *bk, const uint16_t *bv, const uint16_t *norm1,
                         const uint16_t *norm2) {
    sro_layer L = {wq, wk, wv, wo, wg, wu, wd, bq, bk, bv, norm1, norm2};
    m->layers[l] = L;
}

void sro_model_free(sro_model *m) {
    if (!m) return;
    free(m->layers);
    free(m);
}

sro_seq *sro_seq_new(const sro_model *m, int cap) {
    sro_seq *q = (sro_seq *)calloc(1, sizeof(sro_seq));
    size_t n = (size_t)m->s.n_layers * cap * m->s.n_kv_heads * m->s.head_dim;
    q->cap = cap;
    q->k = (real *)calloc(n, sizeof(real));
    q->v = (real *)calloc(n, sizeof(real));
    return q;
}

void sro_seq_free(sro_seq *q) {
    if (!q) return;
    free(q->k);
    free(q->v);
    free(q);
}

int sro_seq_len(const sro_seq *q) { return q->len; }

/* A second sequence with the same tokens behind it (the flat K/V lists are copied). */
sro_seq *sro_seq_clone(const sro_model *m, const sro_seq *q) {
    sro_seq *c = sro_seq_new(m, q->cap);
    const size_t n = (size_t)m->s.n_layers * q->cap * m->s.n_kv_heads * m->s.head_dim;
    memcpy(c->k, q->k, n * sizeof(real));
    memcpy(c->v, q->v, n * sizeof(real));
    c->len = q->len;
    return c;
}
void sro_seq_truncate(sro_seq *q, int len) { if (len < q->len) q->len = len; }

/* y[n] = W[n][:] . x  (+ bias[n]) */
static void matvec(const uint16_t *W, const uint16_t *bias, const real *x, real *y, int N, int K) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        const uint16_t *w = W + (size_t)n * K;
        real acc = 0;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < K; ++k) acc += bf16_to_real(w[k]) * x[k];
        y[n] = bias ? acc + bf16_to_real(bias[n]) : acc;
    }
}

/* RMSNorm: x / sqrt(mean(x^2) + eps) * gain */
static void rmsnorm(const real *x, const uint16_t *gain, real eps, real *y, int H) {
    real ss = 0;
    for (int i = 0; i < H; ++i) ss += x[i] * x[i];
    real inv = (real)1 / (real)sqrt((double)(ss / H + eps));
    for (int i = 0; i < H; ++i) y[i] = rb(x[i] * inv * bf16_to_real(gain[i]));
}

/* Rotate-half RoPE on one head vector at absolute position pos:
 * pair (i, i + d/2), angle = pos * theta^(-2i/d). */
static void rope(real *h, int d, int pos, double theta) {
    const int half = d / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow(theta, -2.0 * i / d);
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = h[i], b = h[i + half];
        h[i] = a * c - b * s;
        h[i + half] = b * c + a * s;
    }
}

/* The same rotation, exported so that tests can pin its convention. */
void sro_rope_apply(real *h, int d, int pos, double theta) { rope(h, d, pos, theta); }

/*
 * Append one token to the sequence: runs every layer at position seq->len,
 * stores its K and V, and (if logits != NULL) writes the vocab logits that
 * predict the next token.  Returns 0, or -1 if the sequence is full.
 */
int sro_forward_token(const sro_model *m, sro_seq *q, int32_t token, real *logits) {
    const sro_shape *s = &m->s;
    const int H = s->hidden, d = s->head_dim, nq = s->n_q_heads, nkv = s->n_kv_heads;
    const int QD = nq * d, KD = nkv * d, F = s->ffn, rep = nq / nkv;
    const int pos = q->len;
    if (pos >= q->cap) return -1;

    real *x = (real *)malloc(sizeof(real) * H);
    real *h = (real *)malloc(sizeof(real) * H);
    real *qv = (real *)malloc(sizeof(real) * QD);
    real *att = (real *)malloc(sizeof(real) * QD);
    real *proj = (real *)malloc(sizeof(real) * H);
    real *g = (real *)malloc(sizeof(real) * F);
    real *u = (real *)malloc(sizeof(real) * F);
    real *sc_all = (real *)malloc(sizeof(real) * (size_t)nq * (pos + 1));   /* one score row per head */

    for (int i = 0; i < H; ++i) x[i] = bf16_to_real(m->embed[(size_t)token * H + i]);

    for (int l = 0; l < s->n_layers; ++l) {
        const sro_layer *L = &m->layers[l];
        real *kc = q->k + ((size_t)l * q->cap) * KD;
        real *vc = q->v + ((size_t)l * q->cap) * KD;
        real *knew = kc + (size_t)pos * KD, *vnew = vc + (size_t)pos * KD;

        rmsnorm(x, L->norm1, (real)s->rms_eps, h, H);
        matvec(L->wq, s->qkv_bias ? L->bq : NULL, h, qv, QD, H);
        matvec(L->wk, s->qkv_bias ? L->bk : NULL, h, knew, KD, H);
        matvec(L->wv, s->qkv_bias ? L->bv : NULL, h, vnew, KD, H);
        for (int a = 0; a < nq; ++a) rope(qv + a * d, d, pos, s->rope_theta);
        for (int a = 0; a < nkv; ++a) rope(knew + a * d, d, pos, s->rope_theta);
        if (g_contract) {
            for (int i = 0; i < QD; ++i) qv[i] = rb(qv[i]);
            for (int i = 0; i < KD; ++i) { knew[i] = rb(knew[i]); vnew[i] = rb(vnew[i]); }
        }

        const real scale = (real)(1.0 / sqrt((double)d));
#pragma omp parallel for schedule(static)
        for (int a = 0; a < nq; ++a) {       /* heads are independent of each other */
            const int kvh = a / rep;
            const real *qa = qv + a * d;
            real *sc = sc_all + (size_t)a * (pos + 1);
            real mx = -INFINITY;
            for (int t = 0; t <= pos; ++t) {
                const real *kt = kc + (size_t)t * KD + kvh * d;
                real dot = 0;
                for (int i = 0; i < d; ++i) dot += qa[i] * kt[i];
                sc[t] = dot * scale;
                if (sc[t] > mx) mx = sc[t];
            }
            real den = 0;
            for (int t = 0; t <= pos; ++t) {
                sc[t] = (real)exp((double)(sc[t] - mx));
                den += sc[t];
            }
            real *oa = att + a * d;
            for (int i = 0; i < d; ++i) oa[i] = 0;
            for (int t = 0; t <= pos; ++t) {
                const real p = rb(sc[t]) / den;
                const real *vt = vc + (size_t)t * KD + kvh * d;
                for (int i = 0; i < d; ++i) oa[i] += p * vt[i];
            }
            if (g_contract)
                for (int i = 0; i < d; ++i) oa[i] = rb(oa[i]);
        }
        matvec(L->wo, NULL, att, proj, H, QD);
        for (int i = 0; i < H; ++i) x[i] += proj[i];

        rmsnorm(x, L->norm2, (real)s->rms_eps, h, H);
        matvec(L->wg, NULL, h, g, F, H);
        matvec(L->wu, NULL, h, u, F, H);
        for (int i = 0; i < F; ++i) {
            real silu = g[i] / ((real)1 + (real)exp((double)-g[i]));
            g[i] = rb(silu * u[i]);
        }
        matvec(L->wd, NULL, g, proj, H, F);
        for (int i = 0; i < H; ++i) x[i] += proj[i];
    }
    q->len = pos + 1;

    if (logits) {
        rmsnorm(x, m->final_norm, (real)s->rms_eps, h, H);
        matvec(m->lm_head, NULL, h, logits, s->vocab, H);
    }
    free(x); free(h); free(qv); free(att); free(proj); free(g); free(u); free(sc_all);
    return 0;
}

/* Append n tokens; logits (if given) are those after the last one. */
int sro_forward(const sro_model *m, sro_seq *q, const int32_t *tokens, int n, real *logits) {
    for (int i = 0; i < n; ++i) {
        int rc = sro_forward_token(m, q, tokens[i], (i == n - 1) ? logits : NULL);
        if (rc) return rc;
    }
    return 0;
}

/*
 * Temperature sampling (the paper's rollouts are sampled at T = 0.7, Section 3.1) by the Gumbel-max
 * rule: token = argmax_v (logit_v / T + g_v) with g_v = -ln(-ln(u_v)) independent standard Gumbel
 * variates, which draws exactly from softmax(logits / T).  The uniforms come from SplitMix64 used
 * counter-based: stream key from (seed, original sequence id, position), counter = vocabulary index,
 * u = (top 23 bits + 0.5) / 2^23.  Lowest index on ties; also reports the gap to the runner-up score.
 */
static uint64_t smx_finalize(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
    return z ^ (z >> 31);
}

int sro_sample(const real *logits, int V, double temperature, uint64_t seed, int32_t orig_seq, int32_t pos,
               double *top2_gap) {
    const uint64_t golden = 0x9E3779B97F4A7C15ULL;
    const uint64_t stream = ((uint64_t)(uint32_t)orig_seq << 32) | (uint32_t)pos;
    const uint64_t key = smx_finalize(smx_finalize(seed + golden) ^ (stream * 0xD1342543DE82EF95ULL + 1ULL));
    int best = 0;
    double best_s = -INFINITY, second = -INFINITY;
    for (int v = 0; v < V; ++v) {
        const uint64_t r = smx_finalize(key + ((uint64_t)v + 1ULL) * golden);
        const double u = ((double)(r >> 41) + 0.5) / 8388608.0;
        const double sc = (double)logits[v] / temperature - log(-log(u));
        if (sc > best_s) { second = best_s; best_s = sc; best = v; }
        else if (sc > second) second = sc;
    }
    if (top2_gap) *top2_gap = best_s - second;
    return best;
}

/* ------------------------------------------------------------------------- */
/* Teacher-forced log-likelihood (Appendix C.2) and the policy-gradient loss   */
/* ------------------------------------------------------------------------- */
/* log softmax(logits)[target]: the largest logit is subtracted before the exponentials. */
double sro_logprob(const real *logits, int V, int32_t target) {
    real mx = logits[0];
    for (int v = 1; v < V; ++v)
        if (logits[v] > mx) mx = logits[v];
    double sum = 0.0;
    for (int v = 0; v < V; ++v) sum += exp((double)(logits[v] - mx));
    return (double)(logits[target] - mx) - log(sum);
}

/*
 * L = -(1/N) sum_i A_i log p(tau_i) over the N = n_groups * G trajectories of the batch, with the
 * group-relative advantages of Eq. 1 (Section 2.1).  logprob, rewards, A: [n_groups][G].
 */
double sro_grpo_loss(const double *logprob, const double *rewards, int n_groups, int G, double eps, double *A) {
    double acc = 0.0;
    for (int g = 0; g < n_groups; ++g) {
        sro_advantage(rewards + (size_t)g * G, G, eps, A + (size_t)g * G);
        for (int i = 0; i < G; ++i) acc += A[(size_t)g * G + i] * logprob[(size_t)g * G + i];
    }
    return -acc / ((double)n_groups * G);
}

/* Greedy choice: lowest index among the maxima.  Also reports the gap to the runner-up. */
int sro_argmax(const real *logits, int V, double *top2_gap) {
    int best = 0;
    for (int v = 1; v < V; ++v)
        if (logits[v] > logits[best]) best = v;
    if (top2_gap) {
        real second = -INFINITY;
        for (int v = 0; v < V; ++v)
            if (v != best && logits[v] > second) second = logits[v];
        *top2_gap = (double)(logits[best] - second);
    }
    return best;
}
