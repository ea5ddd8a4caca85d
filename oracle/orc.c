/*
 * orc.c -- CPU oracle for batched autoregressive generation of a LLaMA-architecture decoder.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU path is checked
 * against.  It shares no code with the GPU library and must never be called from the product path.
 *
 * What it defines (paper, Section 2.1 "RLHF workflow": generation = one prefill forward pass over
 * all prompt tokens that yields the first generated token, then a decode loop that feeds the single
 * latest token and yields the next one; Appendix A "Experiment details": fixed-length prompts, no
 * early stop; model-configuration table: untied input/output embeddings, bias-free projections,
 * NumKVHeads <= NumAttentionHeads, i.e. grouped-query attention):
 *
 *   logits[b, i, :] = f(tokens[b, 0..i])  for every sequence b and position i, f = decoder below,
 *   next token      = argmax of the logits (lowest index on ties).
 *
 * The paper does not print the decoder's internals (it only says "LLaMA models"); the definition
 * used is the standard one:
 *   x = E[token]
 *   per layer:  h = g1 * x / sqrt(mean(x^2) + eps)
 *               q = Wq h, k = Wk h, v = Wv h          (W stored [out, in], no bias)
 *               rotary embedding of every q/k head at the token's absolute position
 *               o_u = softmax_j<=i (q_u . k_{c,j} / sqrt(hd)) v_{c,j},  c = u / (Hq/Hkv)
 *               x += Wo concat(o)
 *               h = g2 * x / sqrt(mean(x^2) + eps);  x += Wd (silu(Wg h) * (Wu h))
 *   logits = Wlm (gf * x / sqrt(mean(x^2) + eps))
 *
 * Arithmetic: all activations, reductions and transcendental functions in fp64.  Weights are given
 * as fp32 values or as bf16 bit patterns and are widened exactly.  There is no blocking, fusion or
 * reordering: orc_forward_all() recomputes everything without any cache; the cached pair
 * orc_prefill()/orc_decode_step() is a second, separately written route to the same numbers and the
 * tests require the two to agree.
 *
 * Threads (OpenMP) split independent outputs only (rows of a projection, (sequence, head) pairs);
 * each output is produced by one thread in a fixed order, so results do not depend on thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t n_layers, hidden, n_heads, n_kv_heads, head_dim, ffn, vocab;
    float rope_base, rms_eps;
    int32_t rope_style;   /* 0: rotate pairs (2r, 2r+1); 1: rotate pairs (r, r + head_dim/2) */
    int32_t weight_dtype; /* 0: fp32 values; 1: bf16 bit patterns (uint16) */
    int32_t max_batch, max_seq;
} orc_shape;

typedef struct {
    const void *tok_emb;
    const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
    const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
    const void *final_norm, *lm_head;
} orc_weights;

typedef struct orc_model {
    orc_shape s;
    orc_weights w;
    const void **ptrs;  /* owned copy of the nine per-layer pointer arrays */
    double *kc, *vc;    /* cache [L][max_batch][max_seq][Hkv*hd] */
    int32_t cur_batch, cur_len;
} orc_model;

enum { ORC_OK = 0, ORC_E_NULL = -1, ORC_E_SHAPE = -2, ORC_E_CAPACITY = -3, ORC_E_STATE = -4, ORC_E_NOMEM = -5 };

/* ------------------------------------------------------------------ scalar helpers */

static double widen_bf16(uint16_t bits) {
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static double weight_at(const void *w, int dtype, size_t idx) {
    return dtype == 0 ? (double)((const float *)w)[idx] : widen_bf16(((const uint16_t *)w)[idx]);
}

static double dot_row(const void *w, int dtype, size_t row, int K, const double *x) {
    double acc = 0.0;
    if (dtype == 0) {
        const float *r = (const float *)w + row * (size_t)K;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < K; ++k) acc += (double)r[k] * x[k];
    } else {
        const uint16_t *r = (const uint16_t *)w + row * (size_t)K;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < K; ++k) acc += widen_bf16(r[k]) * x[k];
    }
    return acc;
}

/* Y[m, n] = sum_k W[n, k] X[m, k]   (W is [N, K] row-major: "out, in") */
void orc_linear(const void *W, int dtype, int N, int K, const double *X, int M, double *Y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int m = 0; m < M; ++m) Y[(size_t)m * N + n] = dot_row(W, dtype, (size_t)n, K, X + (size_t)m * K);
}

/* y = g * x / sqrt(mean(x^2) + eps) */
void orc_rmsnorm(const double *x, const void *g, int gdtype, int d, double eps, double *y) {
    double ss = 0.0;
    for (int j = 0; j < d; ++j) ss += x[j] * x[j];
    double inv = 1.0 / sqrt(ss / (double)d + eps);
    for (int j = 0; j < d; ++j) y[j] = weight_at(g, gdtype, (size_t)j) * x[j] * inv;
}

/* Rotary position embedding of one head vector, in place, at absolute position pos:
 * pair r (0 <= r < hd/2) is rotated by the angle pos * base^(-2r/hd). */
void orc_rope(double *v, int hd, int pos, double base, int style) {
    int half = hd / 2;
    for (int r = 0; r < half; ++r) {
        double theta = pow(base, -2.0 * (double)r / (double)hd);
        double ang = (double)pos * theta;
        double c = cos(ang), s = sin(ang);
        int ia = style == 0 ? 2 * r : r;
        int ib = style == 0 ? 2 * r + 1 : r + half;
        double a = v[ia], b = v[ib];
        v[ia] = a * c - b * s;
        v[ib] = a * s + b * c;
    }
}

/* One query head against n_ctx cached keys/values: o = sum_j softmax_j(q.k_j / sqrt(hd)) v_j.
 * k_j = K + j*stride, v_j = V + j*stride. */
void orc_attend(const double *q, const double *K, const double *V, int n_ctx, int hd, size_t stride, double *o) {
    double *sc = (double *)malloc(sizeof(double) * (size_t)n_ctx);
    double scale = 1.0 / sqrt((double)hd), mx = -INFINITY, den = 0.0;
    for (int j = 0; j < n_ctx; ++j) {
        double a = 0.0;
        for (int e = 0; e < hd; ++e) a += q[e] * K[(size_t)j * stride + e];
        sc[j] = a * scale;
        if (sc[j] > mx) mx = sc[j];
    }
    for (int j = 0; j < n_ctx; ++j) {
        sc[j] = exp(sc[j] - mx);
        den += sc[j];
    }
    for (int e = 0; e < hd; ++e) o[e] = 0.0;
    for (int j = 0; j < n_ctx; ++j) {
        double p = sc[j] / den;
        for (int e = 0; e < hd; ++e) o[e] += p * V[(size_t)j * stride + e];
    }
    free(sc);
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

/* index of the largest value; the lowest index wins ties; -1 if a NaN is present or n <= 0 */
int32_t orc_argmax(const double *x, int n) {
    if (n <= 0) return -1;
    int32_t best = 0;
    for (int i = 0; i < n; ++i) {
        if (x[i] != x[i]) return -1;
        if (x[i] > x[best]) best = i;
    }
    return best;
}

/* Log-probability of one token under the softmax of a logit row (the quantity the inference function call of
 * Section 2.1 returns for every generated token): log p_t = x_t - log sum_v exp(x_v), with the maximum taken out
 * of the exponentials.  NaN if target is outside [0, n). */
double orc_token_logprob(const double *x, int n, int target) {
    if (n <= 0 || target < 0 || target >= n) return NAN;
    double mx = x[0];
    for (int i = 1; i < n; ++i)
        if (x[i] > mx) mx = x[i];
    double sum = 0.0;
    for (int i = 0; i < n; ++i) sum += exp(x[i] - mx);
    return x[target] - (mx + log(sum));
}

/* Temperature sampling by inversion (Section 2.1 samples the next token; the uniform draw u in [0, 1) is an input):
 * p_v = softmax(x / temperature)_v, result = the smallest v with p_0 + ... + p_v > u (the last index with p > 0 if
 * rounding leaves the total at or below u).  -1 for n <= 0, temperature <= 0 or a NaN logit. */
int32_t orc_sample(const double *x, int n, double temperature, double u) {
    if (n <= 0 || !(temperature > 0.0)) return -1;
    double mx = x[0];
    for (int i = 0; i < n; ++i) {
        if (x[i] != x[i]) return -1;
        if (x[i] > mx) mx = x[i];
    }
    double total = 0.0;
    for (int i = 0; i < n; ++i) total += exp((x[i] - mx) / temperature);
    double run = 0.0;
    int32_t last = 0;
    for (int i = 0; i < n; ++i) {
        double p = exp((x[i] - mx) / temperature) / total;
        if (p > 0.0) last = i;
        run += p;
        if (run > u) return i;
    }
    return last;
}

/* ------------------------------------------------------------------ closed forms */

static int shape_ok(const orc_shape *s) {
    if (s->n_layers < 0 || s->hidden <= 0 || s->n_heads <= 0 || s->n_kv_heads <= 0 || s->head_dim <= 0 ||
        s->ffn <= 0 || s->vocab <= 0)
        return 0;
    if (s->n_heads % s->n_kv_heads != 0 || (s->head_dim & 1)) return 0;
    if (s->rope_style != 0 && s->rope_style != 1) return 0;
    if (s->weight_dtype != 0 && s->weight_dtype != 1) return 0;
    return 1;
}

/* Parameter inventory behind the paper's model-configuration table: untied input and output
 * embeddings, Wq and Wo of (Hq*hd) x d, Wk and Wv of (Hkv*hd) x d, three d x F feed-forward
 * matrices, two gain vectors per layer and a final one. */
int64_t orc_param_count(const orc_shape *s) {
    int64_t d = s->hidden, qd = (int64_t)s->n_heads * s->head_dim, kvd = (int64_t)s->n_kv_heads * s->head_dim;
    int64_t per_layer = 2 * qd * d + 2 * kvd * d + 3 * d * (int64_t)s->ffn + 2 * d;
    return 2 * (int64_t)s->vocab * d + (int64_t)s->n_layers * per_layer + d;
}

/* bytes of K and V one token of one sequence occupies when each element takes elem_bytes */
int64_t orc_kv_bytes_per_token(const orc_shape *s, int elem_bytes) {
    return 2LL * s->n_layers * s->n_kv_heads * s->head_dim * elem_bytes;
}

/* ------------------------------------------------------------------ model object */

int orc_create(const orc_shape *s, const orc_weights *w, orc_model **out) {
    if (!s || !w || !out) return ORC_E_NULL;
    if (!shape_ok(s)) return ORC_E_SHAPE;
    if (s->max_batch <= 0 || s->max_seq <= 0) return ORC_E_SHAPE;
    if (!w->tok_emb || !w->final_norm || !w->lm_head) return ORC_E_NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof *m);
    if (!m) return ORC_E_NOMEM;
    m->s = *s;
    int L = s->n_layers;
    m->ptrs = (const void **)calloc((size_t)(9 * (L > 0 ? L : 1)), sizeof(void *));
    const void *const *src[9] = {w->attn_norm, w->wq, w->wk, w->wv, w->wo, w->ffn_norm, w->w_gate, w->w_up, w->w_down};
    for (int a = 0; a < 9; ++a) {
        if (L > 0 && !src[a]) { free(m->ptrs); free(m); return ORC_E_NULL; }
        for (int l = 0; l < L; ++l) {
            if (!src[a][l]) { free(m->ptrs); free(m); return ORC_E_NULL; }
            m->ptrs[a * L + l] = src[a][l];
        }
    }
    m->w = *w;
    m->w.attn_norm = m->ptrs + 0 * L; m->w.wq = m->ptrs + 1 * L; m->w.wk = m->ptrs + 2 * L;
    m->w.wv = m->ptrs + 3 * L; m->w.wo = m->ptrs + 4 * L; m->w.ffn_norm = m->ptrs + 5 * L;
    m->w.w_gate = m->ptrs + 6 * L; m->w.w_up = m->ptrs + 7 * L; m->w.w_down = m->ptrs + 8 * L;
    size_t n = (size_t)(L > 0 ? L : 1) * s->max_batch * s->max_seq * s->n_kv_heads * s->head_dim;
    m->kc = (double *)malloc(n * sizeof(double));
    m->vc = (double *)malloc(n * sizeof(double));
    if (!m->kc || !m->vc) { free(m->kc); free(m->vc); free(m->ptrs); free(m); return ORC_E_NOMEM; }
    m->cur_batch = 0; m->cur_len = 0;
    *out = m;
    return ORC_OK;
}

void orc_destroy(orc_model *m) {
    if (!m) return;
    free(m->kc); free(m->vc); free(m->ptrs); free(m);
}

int orc_reset(orc_model *m) {
    if (!m) return ORC_E_NULL;
    m->cur_batch = 0; m->cur_len = 0;
    return ORC_OK;
}

static void embed(const orc_model *m, int32_t tok, double *x) {
    int d = m->s.hidden;
    for (int j = 0; j < d; ++j) x[j] = weight_at(m->w.tok_emb, m->s.weight_dtype, (size_t)tok * d + j);
}

static int tokens_ok(const orc_model *m, const int32_t *tokens, size_t n) {
    for (size_t i = 0; i < n; ++i)
        if (tokens[i] < 0 || tokens[i] >= m->s.vocab) return 0;
    return 1;
}

/* ------------------------------------------------------------------ the plain definition: no cache
 * tokens [B, T] row-major -> logits [B, T, V].  Every position of every sequence is carried through
 * the layers together; attention at position i looks at positions 0..i of the same sequence. */
int orc_forward_all(const orc_model *m, const int32_t *tokens, int B, int T, double *logits) {
    if (!m || !tokens || !logits) return ORC_E_NULL;
    if (B <= 0 || T <= 0) return ORC_E_SHAPE;
    if (!tokens_ok(m, tokens, (size_t)B * T)) return ORC_E_SHAPE;
    const orc_shape *s = &m->s;
    int d = s->hidden, Hq = s->n_heads, Hkv = s->n_kv_heads, hd = s->head_dim, F = s->ffn, V = s->vocab;
    int qd = Hq * hd, kvd = Hkv * hd, grp = Hq / Hkv, dt = s->weight_dtype;
    size_t M = (size_t)B * T;
    double *x = (double *)malloc(M * d * sizeof(double)), *h = (double *)malloc(M * d * sizeof(double));
    double *q = (double *)malloc(M * qd * sizeof(double)), *k = (double *)malloc(M * kvd * sizeof(double));
    double *v = (double *)malloc(M * kvd * sizeof(double)), *att = (double *)malloc(M * qd * sizeof(double));
    double *y = (double *)malloc(M * d * sizeof(double));
    double *ga = (double *)malloc(M * F * sizeof(double)), *up = (double *)malloc(M * F * sizeof(double));
    if (!x || !h || !q || !k || !v || !att || !y || !ga || !up) {
        free(x); free(h); free(q); free(k); free(v); free(att); free(y); free(ga); free(up);
        return ORC_E_NOMEM;
    }
    for (size_t t = 0; t < M; ++t) embed(m, tokens[t], x + t * d);
    for (int l = 0; l < s->n_layers; ++l) {
        for (size_t t = 0; t < M; ++t) orc_rmsnorm(x + t * d, m->w.attn_norm[l], dt, d, s->rms_eps, h + t * d);
        orc_linear(m->w.wq[l], dt, qd, d, h, (int)M, q);
        orc_linear(m->w.wk[l], dt, kvd, d, h, (int)M, k);
        orc_linear(m->w.wv[l], dt, kvd, d, h, (int)M, v);
        for (size_t t = 0; t < M; ++t) {
            int pos = (int)(t % (size_t)T);
            for (int u = 0; u < Hq; ++u) orc_rope(q + t * qd + (size_t)u * hd, hd, pos, s->rope_base, s->rope_style);
            for (int c = 0; c < Hkv; ++c) orc_rope(k + t * kvd + (size_t)c * hd, hd, pos, s->rope_base, s->rope_style);
        }
#pragma omp parallel for schedule(dynamic)
        for (long bu = 0; bu < (long)B * Hq; ++bu) {
            int b = (int)(bu / Hq), u = (int)(bu % Hq), c = u / grp;
            for (int i = 0; i < T; ++i) {
                size_t t = (size_t)b * T + i;
                /* keys/values of this sequence start at token b*T; causal: i+1 of them are visible */
                orc_attend(q + t * qd + (size_t)u * hd, k + (size_t)b * T * kvd + (size_t)c * hd,
                           v + (size_t)b * T * kvd + (size_t)c * hd, i + 1, hd, (size_t)kvd, att + t * qd + (size_t)u * hd);
            }
        }
        orc_linear(m->w.wo[l], dt, d, qd, att, (int)M, y);
        for (size_t e = 0; e < M * d; ++e) x[e] += y[e];
        for (size_t t = 0; t < M; ++t) orc_rmsnorm(x + t * d, m->w.ffn_norm[l], dt, d, s->rms_eps, h + t * d);
        orc_linear(m->w.w_gate[l], dt, F, d, h, (int)M, ga);
        orc_linear(m->w.w_up[l], dt, F, d, h, (int)M, up);
        for (size_t e = 0; e < M * F; ++e) ga[e] = orc_silu(ga[e]) * up[e];
        orc_linear(m->w.w_down[l], dt, d, F, ga, (int)M, y);
        for (size_t e = 0; e < M * d; ++e) x[e] += y[e];
    }
    for (size_t t = 0; t < M; ++t) orc_rmsnorm(x + t * d, m->w.final_norm, dt, d, s->rms_eps, h + t * d);
    orc_linear(m->w.lm_head, dt, V, d, h, (int)M, logits);
    free(x); free(h); free(q); free(k); free(v); free(att); free(y); free(ga); free(up);
    return ORC_OK;
}

/* ------------------------------------------------------------------ the cached route
 * T new tokens per sequence enter at absolute positions pos0 .. pos0+T-1; their k and v are stored
 * in the cache and the query at position p attends to cache rows 0..p.  Prefill is one such span
 * starting at 0; a decode step is a span of length 1.  tokens is [B, T] row-major.  logits (may be
 * NULL) receives [B, V] for the LAST position of the span. */
static int run_span(orc_model *m, const int32_t *tokens, int B, int T, int pos0, double *logits) {
    const orc_shape *s = &m->s;
    int d = s->hidden, Hq = s->n_heads, Hkv = s->n_kv_heads, hd = s->head_dim, F = s->ffn, V = s->vocab;
    int qd = Hq * hd, kvd = Hkv * hd, grp = Hq / Hkv, dt = s->weight_dtype;
    size_t per_seq = (size_t)s->max_seq * kvd, per_layer = (size_t)s->max_batch * per_seq;
    size_t M = (size_t)B * T;
    double *x = (double *)malloc(M * d * sizeof(double)), *h = (double *)malloc(M * d * sizeof(double));
    double *q = (double *)malloc(M * qd * sizeof(double)), *kk = (double *)malloc(M * kvd * sizeof(double));
    double *vv = (double *)malloc(M * kvd * sizeof(double)), *att = (double *)malloc(M * qd * sizeof(double));
    double *y = (double *)malloc(M * d * sizeof(double));
    double *ga = (double *)malloc(M * F * sizeof(double)), *up = (double *)malloc(M * F * sizeof(double));
    if (!x || !h || !q || !kk || !vv || !att || !y || !ga || !up) {
        free(x); free(h); free(q); free(kk); free(vv); free(att); free(y); free(ga); free(up);
        return ORC_E_NOMEM;
    }
    for (size_t t = 0; t < M; ++t) embed(m, tokens[t], x + t * d);
    for (int l = 0; l < s->n_layers; ++l) {
        for (size_t t = 0; t < M; ++t) orc_rmsnorm(x + t * d, m->w.attn_norm[l], dt, d, s->rms_eps, h + t * d);
        orc_linear(m->w.wq[l], dt, qd, d, h, (int)M, q);
        orc_linear(m->w.wk[l], dt, kvd, d, h, (int)M, kk);
        orc_linear(m->w.wv[l], dt, kvd, d, h, (int)M, vv);
        for (int b = 0; b < B; ++b)
            for (int i = 0; i < T; ++i) {
                size_t t = (size_t)b * T + i;
                int pos = pos0 + i;
                for (int u = 0; u < Hq; ++u) orc_rope(q + t * qd + (size_t)u * hd, hd, pos, s->rope_base, s->rope_style);
                for (int c = 0; c < Hkv; ++c) orc_rope(kk + t * kvd + (size_t)c * hd, hd, pos, s->rope_base, s->rope_style);
                size_t slot = (size_t)l * per_layer + (size_t)b * per_seq + (size_t)pos * kvd;
                memcpy(m->kc + slot, kk + t * kvd, (size_t)kvd * sizeof(double));
                memcpy(m->vc + slot, vv + t * kvd, (size_t)kvd * sizeof(double));
            }
#pragma omp parallel for schedule(dynamic)
        for (long bu = 0; bu < (long)B * Hq; ++bu) {
            int b = (int)(bu / Hq), u = (int)(bu % Hq), c = u / grp;
            const double *Kb = m->kc + (size_t)l * per_layer + (size_t)b * per_seq + (size_t)c * hd;
            const double *Vb = m->vc + (size_t)l * per_layer + (size_t)b * per_seq + (size_t)c * hd;
            for (int i = 0; i < T; ++i) {
                size_t t = (size_t)b * T + i;
                orc_attend(q + t * qd + (size_t)u * hd, Kb, Vb, pos0 + i + 1, hd, (size_t)kvd, att + t * qd + (size_t)u * hd);
            }
        }
        orc_linear(m->w.wo[l], dt, d, qd, att, (int)M, y);
        for (size_t e = 0; e < M * d; ++e) x[e] += y[e];
        for (size_t t = 0; t < M; ++t) orc_rmsnorm(x + t * d, m->w.ffn_norm[l], dt, d, s->rms_eps, h + t * d);
        orc_linear(m->w.w_gate[l], dt, F, d, h, (int)M, ga);
        orc_linear(m->w.w_up[l], dt, F, d, h, (int)M, up);
        for (size_t e = 0; e < M * F; ++e) ga[e] = orc_silu(ga[e]) * up[e];
        orc_linear(m->w.w_down[l], dt, d, F, ga, (int)M, y);
        for (size_t e = 0; e < M * d; ++e) x[e] += y[e];
    }
    if (logits) {
        /* only the last position of each sequence is projected onto the vocabulary */
        for (int b = 0; b < B; ++b) {
            size_t t = (size_t)b * T + (T - 1);
            orc_rmsnorm(x + t * d, m->w.final_norm, dt, d, s->rms_eps, h + (size_t)b * d);
        }
        orc_linear(m->w.lm_head, dt, V, d, h, B, logits);
    }
    free(x); free(h); free(q); free(kk); free(vv); free(att); free(y); free(ga); free(up);
    return ORC_OK;
}

static void greedy(const double *logits, int B, int V, int32_t *next) {
    for (int b = 0; b < B; ++b) next[b] = orc_argmax(logits + (size_t)b * V, V);
}

/* tokens [B, T] -> logits [B, V] of the last prompt position, next [B] = greedy first generated token */
int orc_prefill(orc_model *m, const int32_t *tokens, int B, int T, double *logits, int32_t *next) {
    if (!m || !tokens || !logits) return ORC_E_NULL;
    if (B <= 0 || T <= 0) return ORC_E_SHAPE;
    if (B > m->s.max_batch || T > m->s.max_seq) return ORC_E_CAPACITY;
    if (!tokens_ok(m, tokens, (size_t)B * T)) return ORC_E_SHAPE;
    int rc = run_span(m, tokens, B, T, 0, logits);
    if (rc != ORC_OK) return rc;
    m->cur_batch = B; m->cur_len = T;
    if (next) greedy(logits, B, m->s.vocab, next);
    return ORC_OK;
}

/* tokens [B] (the latest token of each sequence) -> logits [B, V], next [B] */
int orc_decode_step(orc_model *m, const int32_t *tokens, double *logits, int32_t *next) {
    if (!m || !tokens || !logits) return ORC_E_NULL;
    if (m->cur_batch <= 0) return ORC_E_STATE;
    if (m->cur_len + 1 > m->s.max_seq) return ORC_E_CAPACITY;
    if (!tokens_ok(m, tokens, (size_t)m->cur_batch)) return ORC_E_SHAPE;
    int rc = run_span(m, tokens, m->cur_batch, 1, m->cur_len, logits);
    if (rc != ORC_OK) return rc;
    m->cur_len += 1;
    if (next) greedy(logits, m->cur_batch, m->s.vocab, next);
    return ORC_OK;
}

/* tokens [B, T]: T further tokens of each of the current sequences (B must equal the batch of the last orc_prefill), entering
 * at positions cur_len .. cur_len + T - 1 against the cache (Section 2.1: the decode phase consumes tokens against the cache;
 * a span of T > 1 tokens is T consecutive decode steps whose inputs are known beforehand, e.g. a long prompt fed in pieces).
 * logits (may be NULL): [B, V] for the last position of the span. */
int orc_extend(orc_model *m, const int32_t *tokens, int T, double *logits) {
    if (!m || !tokens) return ORC_E_NULL;
    if (m->cur_batch <= 0) return ORC_E_STATE;
    if (T <= 0) return ORC_E_SHAPE;
    if (m->cur_len + T > m->s.max_seq) return ORC_E_CAPACITY;
    if (!tokens_ok(m, tokens, (size_t)m->cur_batch * T)) return ORC_E_SHAPE;
    int rc = run_span(m, tokens, m->cur_batch, T, m->cur_len, logits);
    if (rc != ORC_OK) return rc;
    m->cur_len += T;
    return ORC_OK;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
