/*
 * sanitize_check.c -- drives every entry point of orc.c on tiny models under AddressSanitizer and
 * UndefinedBehaviorSanitizer (CPU only).  TEST INFRASTRUCTURE ONLY, like orc.c itself: built by
 * oracle/build.py:build_sanitize_check() as a stand-alone executable that links orc.c directly, run by
 * the CPU test suite.  It checks memory and arithmetic hygiene (every access in bounds at ragged
 * shapes, every error path free of leaks and overflows), not values: the values are pinned elsewhere.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, hidden, n_heads, n_kv_heads, head_dim, ffn, vocab;
    float rope_base, rms_eps;
    int32_t rope_style, weight_dtype, max_batch, max_seq;
} orc_shape;
typedef struct {
    const void *tok_emb;
    const void *const *attn_norm, *const *wq, *const *wk, *const *wv, *const *wo;
    const void *const *ffn_norm, *const *w_gate, *const *w_up, *const *w_down;
    const void *final_norm, *lm_head;
} orc_weights;
typedef struct orc_model orc_model;

void orc_linear(const void *W, int dtype, int N, int K, const double *X, int M, double *Y);
void orc_rmsnorm(const double *x, const void *g, int gdtype, int d, double eps, double *y);
void orc_rope(double *v, int hd, int pos, double base, int style);
void orc_attend(const double *q, const double *K, const double *V, int n_ctx, int hd, size_t stride, double *o);
double orc_silu(double z);
int32_t orc_argmax(const double *x, int n);
double orc_token_logprob(const double *x, int n, int target);
int32_t orc_sample(const double *x, int n, double temperature, double u);
int64_t orc_param_count(const orc_shape *s);
int64_t orc_kv_bytes_per_token(const orc_shape *s, int elem_bytes);
int orc_create(const orc_shape *s, const orc_weights *w, orc_model **out);
void orc_destroy(orc_model *m);
int orc_reset(orc_model *m);
int orc_forward_all(const orc_model *m, const int32_t *tokens, int B, int T, double *logits);
int orc_prefill(orc_model *m, const int32_t *tokens, int B, int T, double *logits, int32_t *next);
int orc_decode_step(orc_model *m, const int32_t *tokens, double *logits, int32_t *next);
int orc_extend(orc_model *m, const int32_t *tokens, int T, double *logits);
int orc_num_threads(void);

static uint64_t rng_state = 0x243F6A8885A308D3ull;
static double uniform(void) {  /* xorshift64*: inputs only */
    rng_state ^= rng_state >> 12; rng_state ^= rng_state << 25; rng_state ^= rng_state >> 27;
    return (double)((rng_state * 0x2545F4914F6CDD1Dull) >> 11) / 9007199254740992.0;
}
static float small(void) { return (float)((uniform() - 0.5) * 0.2); }

static uint16_t to_bf16_bits(float f) {  /* truncation is enough here: any bit pattern is a valid input */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

/* exactly-sized allocations so that an access one element out of bounds is caught */
static void *tensor(size_t n, int dtype, int gain) {
    if (dtype == 0) {
        float *p = (float *)malloc(n * sizeof(float));
        for (size_t i = 0; i < n; ++i) p[i] = gain ? 1.0f + small() : small();
        return p;
    }
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) p[i] = to_bf16_bits(gain ? 1.0f + small() : small());
    return p;
}

#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) { fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); exit(1); } \
    } while (0)

static void run_model(int L, int d, int Hq, int Hkv, int hd, int F, int V, int style, int dtype, int B, int P, int G) {
    orc_shape s = {L, d, Hq, Hkv, hd, F, V, 10000.0f, 1e-5f, style, dtype, B, P + G};
    const int qd = Hq * hd, kvd = Hkv * hd;
    const int nl = L > 0 ? L : 1;
    void **lw[9];
    const size_t sizes[9] = {(size_t)d, (size_t)qd * d, (size_t)kvd * d, (size_t)kvd * d, (size_t)d * qd,
                             (size_t)d, (size_t)F * d, (size_t)F * d, (size_t)d * F};
    for (int a = 0; a < 9; ++a) {
        lw[a] = (void **)malloc(nl * sizeof(void *));
        for (int l = 0; l < L; ++l) lw[a][l] = tensor(sizes[a], dtype, a == 0 || a == 5);
    }
    orc_weights w;
    w.tok_emb = tensor((size_t)V * d, dtype, 0);
    w.final_norm = tensor((size_t)d, dtype, 1);
    w.lm_head = tensor((size_t)V * d, dtype, 0);
    w.attn_norm = (const void *const *)lw[0]; w.wq = (const void *const *)lw[1]; w.wk = (const void *const *)lw[2];
    w.wv = (const void *const *)lw[3]; w.wo = (const void *const *)lw[4]; w.ffn_norm = (const void *const *)lw[5];
    w.w_gate = (const void *const *)lw[6]; w.w_up = (const void *const *)lw[7]; w.w_down = (const void *const *)lw[8];

    CHECK(orc_param_count(&s) > 0 && orc_kv_bytes_per_token(&s, 2) == 4LL * L * kvd);
    orc_model *m = NULL;
    CHECK(orc_create(&s, &w, &m) == 0 && m);

    const int T = P + G;
    int32_t *tok = (int32_t *)malloc((size_t)B * T * sizeof(int32_t));
    for (int i = 0; i < B * T; ++i) tok[i] = (int32_t)(uniform() * V) % V;
    double *all = (double *)malloc((size_t)B * T * V * sizeof(double));
    CHECK(orc_forward_all(m, tok, B, T, all) == 0);

    /* cached route: prefill of P tokens, one span of G - 1 tokens, one single step; last logits must match the plain route */
    int32_t *prompt = (int32_t *)malloc((size_t)B * P * sizeof(int32_t));
    for (int b = 0; b < B; ++b) memcpy(prompt + (size_t)b * P, tok + (size_t)b * T, P * sizeof(int32_t));
    double *lg = (double *)malloc((size_t)B * V * sizeof(double));
    int32_t *next = (int32_t *)malloc(B * sizeof(int32_t));
    CHECK(orc_decode_step(m, tok, lg, next) == -4);  /* no prefill yet */
    CHECK(orc_prefill(m, prompt, B, P, lg, next) == 0);
    if (G > 1) {
        int32_t *span = (int32_t *)malloc((size_t)B * (G - 1) * sizeof(int32_t));
        for (int b = 0; b < B; ++b) memcpy(span + (size_t)b * (G - 1), tok + (size_t)b * T + P, (G - 1) * sizeof(int32_t));
        CHECK(orc_extend(m, span, G - 1, NULL) == 0);
        free(span);
    }
    int32_t *last = (int32_t *)malloc(B * sizeof(int32_t));
    for (int b = 0; b < B; ++b) last[b] = tok[(size_t)b * T + T - 1];
    CHECK(orc_decode_step(m, last, lg, next) == 0);
    for (int b = 0; b < B; ++b)
        for (int v = 0; v < V; ++v) {
            double a = lg[(size_t)b * V + v], e = all[((size_t)b * T + T - 1) * V + v];
            CHECK(fabs(a - e) <= 1e-9 * (1.0 + fabs(e)));
        }
    for (int b = 0; b < B; ++b) CHECK(next[b] == orc_argmax(lg + (size_t)b * V, V));
    CHECK(orc_decode_step(m, last, lg, next) == -3);        /* the cache is full */
    CHECK(orc_extend(m, last, 1, NULL) == -3);
    CHECK(orc_reset(m) == 0);
    CHECK(orc_prefill(m, prompt, B + 1, P, lg, next) == -3); /* more sequences than reserved */
    tok[0] = V;                                              /* a token outside the vocabulary is refused, not read */
    CHECK(orc_forward_all(m, tok, B, T, all) == -2);
    tok[0] = -1;
    CHECK(orc_prefill(m, tok, 1, 1, lg, next) == -2);

    orc_destroy(m);
    free(last); free(next); free(lg); free(prompt); free(all); free(tok);
    for (int a = 0; a < 9; ++a) {
        for (int l = 0; l < L; ++l) free(lw[a][l]);
        free(lw[a]);
    }
    free((void *)w.tok_emb); free((void *)w.final_norm); free((void *)w.lm_head);
}

static void run_functions(void) {
    enum { N = 7, K = 13, M = 3, HD = 6, CTX = 5 };
    float *W = (float *)malloc(N * K * sizeof(float));
    double *X = (double *)malloc(M * K * sizeof(double)), *Y = (double *)malloc(M * N * sizeof(double));
    for (int i = 0; i < N * K; ++i) W[i] = small();
    for (int i = 0; i < M * K; ++i) X[i] = small();
    orc_linear(W, 0, N, K, X, M, Y);
    uint16_t *Wb = (uint16_t *)malloc(N * K * sizeof(uint16_t));
    for (int i = 0; i < N * K; ++i) Wb[i] = to_bf16_bits(W[i]);
    orc_linear(Wb, 1, N, K, X, M, Y);
    float *g = (float *)malloc(K * sizeof(float));
    for (int i = 0; i < K; ++i) g[i] = 1.0f + small();
    double *y = (double *)malloc(K * sizeof(double));
    orc_rmsnorm(X, g, 0, K, 1e-5, y);
    double *v = (double *)malloc(HD * sizeof(double));
    for (int style = 0; style < 2; ++style) {
        for (int i = 0; i < HD; ++i) v[i] = small();
        orc_rope(v, HD, 4095, 10000.0, style);
    }
    /* K and V rows with a stride larger than the head: the last row ends exactly at the end of the allocation */
    const size_t stride = HD + 3;
    double *Kc = (double *)malloc(((CTX - 1) * stride + HD) * sizeof(double));
    double *Vc = (double *)malloc(((CTX - 1) * stride + HD) * sizeof(double));
    for (size_t i = 0; i < (CTX - 1) * stride + HD; ++i) { Kc[i] = small(); Vc[i] = small(); }
    double *o = (double *)malloc(HD * sizeof(double));
    orc_attend(v, Kc, Vc, CTX, HD, stride, o);
    orc_attend(v, Kc, Vc, 1, HD, stride, o);
    CHECK(orc_silu(0.0) == 0.0 && orc_silu(-800.0) == 0.0 && orc_silu(800.0) == 800.0);
    double lg[4] = {0.5, -1e300, 1e300, 0.25};
    CHECK(orc_argmax(lg, 4) == 2 && orc_argmax(lg, 0) == -1);
    CHECK(orc_token_logprob(lg, 4, 2) == 0.0);
    CHECK(orc_sample(lg, 4, 1.0, 0.999) == 2 && orc_sample(lg, 4, 0.0, 0.5) == -1 && orc_sample(lg, 0, 1.0, 0.5) == -1);
    lg[1] = NAN;
    CHECK(orc_argmax(lg, 4) == -1 && orc_sample(lg, 4, 1.0, 0.5) == -1);
    CHECK(orc_num_threads() >= 1);
    free(o); free(Vc); free(Kc); free(v); free(y); free(g); free(Wb); free(Y); free(X); free(W);
}

int main(void) {
    run_functions();
    /* L, d, Hq, Hkv, hd, F, V, rope style, weight dtype, B, P, G */
    run_model(2, 24, 4, 2, 6, 40, 37, 1, 1, 3, 5, 4);   /* grouped-query, bf16 bit patterns, ragged sizes */
    run_model(1, 16, 2, 2, 8, 24, 19, 0, 0, 2, 1, 1);   /* fp32 values, interleaved pairs, one-token prompt, no span */
    run_model(0, 8, 2, 1, 4, 8, 11, 1, 1, 1, 3, 2);     /* no layers */
    /* refusals that must free what they allocated */
    orc_shape bad = {1, 8, 3, 2, 4, 8, 11, 10000.0f, 1e-5f, 1, 1, 1, 4};
    orc_weights none;
    memset(&none, 0, sizeof none);
    orc_model *m = NULL;
    CHECK(orc_create(&bad, &none, &m) == -2);
    bad.n_heads = 2;
    CHECK(orc_create(&bad, &none, &m) == -1 && orc_create(NULL, &none, &m) == -1);
    CHECK(orc_reset(NULL) == -1);
    orc_destroy(NULL);
    puts("orc sanitize check: ok");
    return 0;
}
