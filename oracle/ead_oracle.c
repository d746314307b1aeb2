/*
 * CPU oracle for Entropy Adaptive Decoding -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the decode path
 * computes, written from the paper's definitions (Section 3.1, Eq. 1-3;
 * Section 3.2, Eq. 4; Algorithm 1) over a pre-norm decoder-only transformer
 * (RMSNorm, rotary embedding, grouped-query attention, SwiGLU).  It shares no
 * code with the GPU library and is never called by it; only the tests, the
 * smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Precision: tensors are stored as float (the weights it is given are the exact
 * values the GPU path receives, up-cast to float); every long reduction (dot
 * products, vocabulary sums, softmax normalisers) accumulates in double.  The
 * gate arithmetic (window mean, threshold compare) is done in float because it
 * decides an integer: both sides of a parity test must round it identically.
 *
 * No blocking, fusion or reordering: each function is the definition written
 * out as loops.  OpenMP only spreads independent output elements over cores.
 *
 * Parity pins (see tests/): entropy closed forms and brute force; window mean
 * brute force; hand-derived gate traces; the parameter-ratio column of the
 * paper's Table 1; the forward pass against an independent float64 NumPy
 * derivation, its single-token closed form, causality, rotary invariants and
 * the cached-vs-dense identity; the sampler against the generator's published
 * known-answer vectors, an independent integer re-implementation, chi-square
 * tests of sampled frequencies against softmax(l/T), and its T -> 0 limit.  The paper's accuracy claims (benchmark scores,
 * best threshold range) need its dataset and trained weights: parity unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_SMALL 0
#define ORACLE_LARGE 1
#define ORACLE_NATS 0
#define ORACLE_BITS 1

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rms_eps, rope_theta;
    const float *embed;                 /* [vocab, d]              */
    const float *const *wq;             /* per layer [H*hd, d]     */
    const float *const *wk;             /* per layer [KV*hd, d]    */
    const float *const *wv;             /* per layer [KV*hd, d]    */
    const float *const *wo;             /* per layer [d, H*hd]     */
    const float *const *w_gate;         /* per layer [F, d]        */
    const float *const *w_up;           /* per layer [F, d]        */
    const float *const *w_down;         /* per layer [d, F]        */
    const float *const *norm_attn;      /* per layer [d]           */
    const float *const *norm_ffn;       /* per layer [d]           */
    const float *norm_final;            /* [d]                     */
    const float *lm_head;               /* [vocab, d]              */
} oracle_model;

/* ------------------------------------------------------------------------- */
/* Eq. 1-2: softmax of the raw logits, then Shannon entropy.                  */
/* With m = max l, Z = sum exp(l-m), S = sum exp(l-m)(l-m):                   */
/*   -sum p ln p = ln Z - S/Z   (terms with p = 0 contribute 0).              */
/* The paper writes log2; unit selects bits (its Eq. 2) or nats.              */
/* argmax: smallest index attaining the maximum (greedy decoding).            */
/* ------------------------------------------------------------------------- */
double oracle_entropy(const float *l, int32_t V, int32_t unit, int32_t *argmax_out)
{
    float m = l[0];
    int32_t am = 0;
    for (int32_t i = 1; i < V; ++i)
        if (l[i] > m) { m = l[i]; am = i; }
    double Z = 0.0, S = 0.0;
    for (int32_t i = 0; i < V; ++i) {
        double d = (double)l[i] - (double)m;
        double e = exp(d);
        Z += e;
        if (e > 0.0) S += e * d;
    }
    double H = log(Z) - S / Z;
    if (unit == ORACLE_BITS) H /= log(2.0);
    if (argmax_out) *argmax_out = am;
    return H;
}

/* Direct form of Eq. 1-2, -sum p log p, used to cross-check the above. */
double oracle_entropy_direct(const float *l, int32_t V, int32_t unit)
{
    double m = l[0];
    for (int32_t i = 1; i < V; ++i) if (l[i] > m) m = l[i];
    double Z = 0.0;
    for (int32_t i = 0; i < V; ++i) Z += exp((double)l[i] - m);
    double H = 0.0;
    for (int32_t i = 0; i < V; ++i) {
        double p = exp((double)l[i] - m) / Z;
        if (p > 0.0) H -= p * log(p);
    }
    return unit == ORACLE_BITS ? H / log(2.0) : H;
}

/* ------------------------------------------------------------------------- */
/* Eq. 3 as Algorithm 1 states it: mean of the last min(t, w) entries of the  */
/* entropy list W (t = entries so far), summed oldest to newest, in float.    */
/* ------------------------------------------------------------------------- */
float oracle_window_mean(const float *W, int32_t t, int32_t w)
{
    int32_t n = t < w ? t : w;
    float s = 0.0f;
    for (int32_t i = t - n; i < t; ++i) s = s + W[i];
    return s / (float)n;
}

/* ------------------------------------------------------------------------- */
/* Eq. 4 / the switching block of Algorithm 1.  Called after a token has been */
/* emitted: c counts tokens by the current model; a switch needs c >= d_min.  */
/* ------------------------------------------------------------------------- */
void oracle_gate_step(int32_t *model, int32_t *c, float Hbar, float tau, int32_t d_min)
{
    *c = *c + 1;
    if (*c >= d_min) {
        if (*model == ORACLE_SMALL && Hbar > tau) { *model = ORACLE_LARGE; *c = 0; }
        else if (*model == ORACLE_LARGE && Hbar <= tau) { *model = ORACLE_SMALL; *c = 0; }
    }
}

/* Gate driven by a given entropy trace H[0..n): ids[t] = model that produced */
/* token t, Hbar[t] = window mean after appending H[t].                        */
void oracle_gate_trace(const float *H, int32_t n, int32_t w, int32_t d_min, float tau,
                       float *Hbar_out, uint8_t *ids_out)
{
    int32_t model = ORACLE_SMALL, c = 0;
    for (int32_t t = 0; t < n; ++t) {
        float hb = oracle_window_mean(H, t + 1, w);
        if (Hbar_out) Hbar_out[t] = hb;
        ids_out[t] = (uint8_t)model;
        oracle_gate_step(&model, &c, hb, tau, d_min);
    }
}

/* Footnote of Table 1: average parameters per forward pass relative to the   */
/* large model, (alpha P_S + beta P_L) / P_L with beta = large-model share.   */
double oracle_param_ratio(double large_share, double P_S, double P_L)
{
    return ((1.0 - large_share) * P_S + large_share * P_L) / P_L;
}

/* ------------------------------------------------------------------------- */
/* Transformer pieces                                                         */
/* ------------------------------------------------------------------------- */
void oracle_rmsnorm(const float *x, const float *g, int32_t d, float eps, float *out)
{
    double ss = 0.0;
    for (int32_t i = 0; i < d; ++i) ss += (double)x[i] * (double)x[i];
    double r = 1.0 / sqrt(ss / (double)d + (double)eps);
    for (int32_t i = 0; i < d; ++i) out[i] = (float)((double)x[i] * r * (double)g[i]);
}

/* y[n] = sum_k W[n,k] x[k]  (W row-major [N,K]); add != 0 accumulates into y */
void oracle_matvec(const float *W, const float *x, int32_t N, int32_t K, float *y, int32_t add)
{
#pragma omp parallel for schedule(static)
    for (int32_t n = 0; n < N; ++n) {
        const float *wr = W + (size_t)n * (size_t)K;
        double acc = 0.0;
        for (int32_t k = 0; k < K; ++k) acc += (double)wr[k] * (double)x[k];
        y[n] = add ? (float)((double)y[n] + acc) : (float)acc;
    }
}

/* Rotary embedding, "rotate-half" pairing: within a head of width hd, element */
/* i < hd/2 pairs with i + hd/2 and the pair turns by pos * theta^(-2i/hd).    */
void oracle_rope(float *v, int32_t n_heads, int32_t hd, int32_t pos, float theta)
{
    int32_t half = hd / 2;
    for (int32_t h = 0; h < n_heads; ++h) {
        float *p = v + (size_t)h * hd;
        for (int32_t i = 0; i < half; ++i) {
            double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)hd);
            double c = cos(ang), s = sin(ang);
            double a = p[i], b = p[i + half];
            p[i] = (float)(a * c - b * s);
            p[i + half] = (float)(a * s + b * c);
        }
    }
}

static double silu(double x) { return x / (1.0 + exp(-x)); }

/* Attention of ONE query position over keys/values 0..n_keys-1.             */
/* q: [H*hd]; K, V: [n_keys][KV*hd] with row stride kv_stride floats.         */
/* Query head h reads KV head h / (H/KV).  out: [H*hd].                       */
static void attend_one(const oracle_model *m, const float *q, const float *K, const float *V,
                       size_t kv_stride, int32_t n_keys, float *out, double *score)
{
    int32_t hd = m->head_dim, group = m->n_heads / m->n_kv_heads;
    double scale = 1.0 / sqrt((double)hd);
    for (int32_t h = 0; h < m->n_heads; ++h) {
        int32_t kvh = h / group;
        const float *qh = q + (size_t)h * hd;
        double mx = -INFINITY;
        for (int32_t j = 0; j < n_keys; ++j) {
            const float *kj = K + (size_t)j * kv_stride + (size_t)kvh * hd;
            double s = 0.0;
            for (int32_t i = 0; i < hd; ++i) s += (double)qh[i] * (double)kj[i];
            s *= scale;
            score[j] = s;
            if (s > mx) mx = s;
        }
        double Z = 0.0;
        for (int32_t j = 0; j < n_keys; ++j) { score[j] = exp(score[j] - mx); Z += score[j]; }
        for (int32_t i = 0; i < hd; ++i) {
            double acc = 0.0;
            for (int32_t j = 0; j < n_keys; ++j)
                acc += score[j] * (double)V[(size_t)j * kv_stride + (size_t)kvh * hd + i];
            out[(size_t)h * hd + i] = (float)(acc / Z);
        }
    }
}

/* ------------------------------------------------------------------------- */
/* KV-cached incremental forward                                              */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t max_seq, n_layers, kv_width;   /* kv_width = KV*hd */
    int32_t len;                           /* positions filled */
    float *k, *v;                          /* [L][max_seq][kv_width] */
} oracle_cache;

oracle_cache *oracle_cache_new(const oracle_model *m, int32_t max_seq)
{
    oracle_cache *c = (oracle_cache *)calloc(1, sizeof(*c));
    if (!c) return NULL;
    c->max_seq = max_seq; c->n_layers = m->n_layers; c->kv_width = m->n_kv_heads * m->head_dim;
    size_t n = (size_t)m->n_layers * max_seq * c->kv_width;
    c->k = (float *)calloc(n, sizeof(float));
    c->v = (float *)calloc(n, sizeof(float));
    if (!c->k || !c->v) { free(c->k); free(c->v); free(c); return NULL; }
    return c;
}
void oracle_cache_free(oracle_cache *c) { if (c) { free(c->k); free(c->v); free(c); } }
void oracle_cache_reset(oracle_cache *c) { c->len = 0; }
int32_t oracle_cache_len(const oracle_cache *c) { return c->len; }

/* Feed one token at position cache->len; logits (may be NULL) gets [vocab].  */
/* Returns 0, or -1 if the cache is full / the token is out of range.         */
int32_t oracle_forward_cached(const oracle_model *m, oracle_cache *c, int32_t token, float *logits)
{
    int32_t d = m->d_model, hd = m->head_dim, qw = m->n_heads * hd, kw = c->kv_width, F = m->d_ffn;
    int32_t pos = c->len;
    if (pos >= c->max_seq || token < 0 || token >= m->vocab) return -1;
    float *x = (float *)malloc(sizeof(float) * d), *a = (float *)malloc(sizeof(float) * d);
    float *q = (float *)malloc(sizeof(float) * qw), *o = (float *)malloc(sizeof(float) * qw);
    float *g = (float *)malloc(sizeof(float) * F), *u = (float *)malloc(sizeof(float) * F);
    double *score = (double *)malloc(sizeof(double) * (pos + 1));
    memcpy(x, m->embed + (size_t)token * d, sizeof(float) * d);
    for (int32_t l = 0; l < m->n_layers; ++l) {
        float *kc = c->k + ((size_t)l * c->max_seq) * kw, *vc = c->v + ((size_t)l * c->max_seq) * kw;
        oracle_rmsnorm(x, m->norm_attn[l], d, m->rms_eps, a);
        oracle_matvec(m->wq[l], a, qw, d, q, 0);
        oracle_matvec(m->wk[l], a, kw, d, kc + (size_t)pos * kw, 0);
        oracle_matvec(m->wv[l], a, kw, d, vc + (size_t)pos * kw, 0);
        oracle_rope(q, m->n_heads, hd, pos, m->rope_theta);
        oracle_rope(kc + (size_t)pos * kw, m->n_kv_heads, hd, pos, m->rope_theta);
        attend_one(m, q, kc, vc, (size_t)kw, pos + 1, o, score);
        oracle_matvec(m->wo[l], o, d, qw, x, 1);
        oracle_rmsnorm(x, m->norm_ffn[l], d, m->rms_eps, a);
        oracle_matvec(m->w_gate[l], a, F, d, g, 0);
        oracle_matvec(m->w_up[l], a, F, d, u, 0);
        for (int32_t i = 0; i < F; ++i) g[i] = (float)(silu((double)g[i]) * (double)u[i]);
        oracle_matvec(m->w_down[l], g, d, F, x, 1);
    }
    c->len = pos + 1;
    if (logits) {
        oracle_rmsnorm(x, m->norm_final, d, m->rms_eps, a);
        oracle_matvec(m->lm_head, a, m->vocab, d, logits, 0);
    }
    free(x); free(a); free(q); free(o); free(g); free(u); free(score);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Dense forward: the whole sequence at once, explicit causal attention.      */
/* logits: [T][vocab].  Independent of the cached path except for the small   */
/* per-vector helpers above.                                                  */
/* ------------------------------------------------------------------------- */
int32_t oracle_forward_dense(const oracle_model *m, const int32_t *tokens, int32_t T, float *logits)
{
    int32_t d = m->d_model, hd = m->head_dim, qw = m->n_heads * hd, kw = m->n_kv_heads * hd, F = m->d_ffn;
    for (int32_t t = 0; t < T; ++t) if (tokens[t] < 0 || tokens[t] >= m->vocab) return -1;
    float *X = (float *)malloc(sizeof(float) * (size_t)T * d), *A = (float *)malloc(sizeof(float) * (size_t)T * d);
    float *Q = (float *)malloc(sizeof(float) * (size_t)T * qw), *O = (float *)malloc(sizeof(float) * (size_t)T * qw);
    float *Kk = (float *)malloc(sizeof(float) * (size_t)T * kw), *Vv = (float *)malloc(sizeof(float) * (size_t)T * kw);
    float *G = (float *)malloc(sizeof(float) * (size_t)T * F), *U = (float *)malloc(sizeof(float) * (size_t)T * F);
    for (int32_t t = 0; t < T; ++t) memcpy(X + (size_t)t * d, m->embed + (size_t)tokens[t] * d, sizeof(float) * d);
    for (int32_t l = 0; l < m->n_layers; ++l) {
        for (int32_t t = 0; t < T; ++t) {
            oracle_rmsnorm(X + (size_t)t * d, m->norm_attn[l], d, m->rms_eps, A + (size_t)t * d);
            oracle_matvec(m->wq[l], A + (size_t)t * d, qw, d, Q + (size_t)t * qw, 0);
            oracle_matvec(m->wk[l], A + (size_t)t * d, kw, d, Kk + (size_t)t * kw, 0);
            oracle_matvec(m->wv[l], A + (size_t)t * d, kw, d, Vv + (size_t)t * kw, 0);
            oracle_rope(Q + (size_t)t * qw, m->n_heads, hd, t, m->rope_theta);
            oracle_rope(Kk + (size_t)t * kw, m->n_kv_heads, hd, t, m->rope_theta);
        }
#pragma omp parallel
        {
            double *score = (double *)malloc(sizeof(double) * T);
#pragma omp for schedule(dynamic)
            for (int32_t t = 0; t < T; ++t)   /* causal: position t sees keys 0..t */
                attend_one(m, Q + (size_t)t * qw, Kk, Vv, (size_t)kw, t + 1, O + (size_t)t * qw, score);
            free(score);
        }
        for (int32_t t = 0; t < T; ++t) {
            oracle_matvec(m->wo[l], O + (size_t)t * qw, d, qw, X + (size_t)t * d, 1);
            oracle_rmsnorm(X + (size_t)t * d, m->norm_ffn[l], d, m->rms_eps, A + (size_t)t * d);
            oracle_matvec(m->w_gate[l], A + (size_t)t * d, F, d, G + (size_t)t * F, 0);
            oracle_matvec(m->w_up[l], A + (size_t)t * d, F, d, U + (size_t)t * F, 0);
            for (int32_t i = 0; i < F; ++i)
                G[(size_t)t * F + i] = (float)(silu((double)G[(size_t)t * F + i]) * (double)U[(size_t)t * F + i]);
            oracle_matvec(m->w_down[l], G + (size_t)t * F, d, F, X + (size_t)t * d, 1);
        }
    }
    for (int32_t t = 0; t < T; ++t) {
        oracle_rmsnorm(X + (size_t)t * d, m->norm_final, d, m->rms_eps, A + (size_t)t * d);
        oracle_matvec(m->lm_head, A + (size_t)t * d, m->vocab, d, logits + (size_t)t * m->vocab, 0);
    }
    free(X); free(A); free(Q); free(O); free(Kk); free(Vv); free(G); free(U);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1's sampling step: y ~ softmax(l / T) (temperature T > 0).       */
/* Written as the Gumbel-max identity: with u_i independent uniforms on (0,1) */
/* and g_i = -ln(-ln u_i), argmax_i (l_i / T + g_i) is distributed exactly as */
/* softmax(l / T).  The entropy of Eq. 1-2 is still taken from the raw logits.*/
/*                                                                            */
/* The uniforms come from a counter-based generator, so that a draw is a pure */
/* function of (seed, sequence, token index, vocabulary index) and needs no   */
/* state: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, "Parallel   */
/* random numbers: as easy as 1, 2, 3", SC 2011).  One round maps the counter */
/* (c0,c1,c2,c3) under the key (k0,k1) to                                     */
/*   (hi(M1*c2) ^ c1 ^ k0, lo(M1*c2), hi(M0*c0) ^ c3 ^ k1, lo(M0*c0))         */
/* and the key is bumped by the Weyl constants between rounds.                */
/* key = the 64-bit seed; counter = (i / 4, token index, sequence index, 0);  */
/* logit i uses output word i % 4.  u = (2k + 1) / 2^24 with k the top 23     */
/* bits of the word: strictly inside (0, 1) and exact in float.               */
/* The score l/T + g is formed in float with one fused multiply-add, because  */
/* it decides an integer: both sides of a parity test must round it alike.    */
/* ------------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = M0 * c0, p1 = M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

float oracle_uniform(uint64_t seed, int32_t seq_index, int32_t token_index, int32_t i)
{
    uint32_t ctr[4] = { (uint32_t)i >> 2, (uint32_t)token_index, (uint32_t)seq_index, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) }, out[4];
    oracle_philox4x32_10(ctr, key, out);
    uint32_t k = out[i & 3] >> 9;
    return (float)(2u * k + 1u) * (1.0f / 16777216.0f);
}

float oracle_gumbel(uint64_t seed, int32_t seq_index, int32_t token_index, int32_t i)
{
    return -logf(-logf(oracle_uniform(seed, seq_index, token_index, i)));
}

/* y ~ softmax(l / T); T <= 0 selects greedy decoding.  Lowest index on ties. */
int32_t oracle_sample(const float *l, int32_t V, float temperature, uint64_t seed,
                      int32_t seq_index, int32_t token_index)
{
    int32_t best = 0;
    if (!(temperature > 0.0f)) {
        for (int32_t i = 1; i < V; ++i) if (l[i] > l[best]) best = i;
        return best;
    }
    const float inv_t = 1.0f / temperature;
    float bs = -INFINITY;
    for (int32_t i = 0; i < V; ++i) {
        float s = fmaf(l[i], inv_t, oracle_gumbel(seed, seq_index, token_index, i));
        if (s > bs) { bs = s; best = i; }
    }
    return best;
}

/* ------------------------------------------------------------------------- */
/* Algorithm 1.  temperature <= 0: greedy (token = argmax of the raw logits); */
/* otherwise the token is sampled as above (seq_index tells batch rows apart).*/
/* Each model conditions on the whole sequence x + y: a model that was idle   */
/* first consumes the tokens it has not seen (no entropy is recorded there).  */
/* Outputs have room for max_new entries; returns the number generated, or    */
/* a negative value on error.                                                 */
/* ------------------------------------------------------------------------- */
int32_t oracle_generate_sampled(const oracle_model *small, const oracle_model *large,
                                const int32_t *prompt, int32_t n_prompt, int32_t max_new,
                                int32_t w, float tau, int32_t d_min, int32_t unit, int32_t eos_id,
                                float temperature, uint64_t seed, int32_t seq_index,
                                int32_t *out_tokens, uint8_t *out_model, float *out_H, float *out_Hbar)
{
    if (small->vocab != large->vocab || n_prompt < 1 || w < 1 || d_min < 1) return -1;
    int32_t V = small->vocab, total = n_prompt + max_new;
    const oracle_model *mdl[2] = { small, large };
    oracle_cache *cache[2] = { oracle_cache_new(small, total), oracle_cache_new(large, total) };
    int32_t *seq = (int32_t *)malloc(sizeof(int32_t) * total);
    float *logits = (float *)malloc(sizeof(float) * V);
    float *W = (float *)malloc(sizeof(float) * (max_new > 0 ? max_new : 1));
    memcpy(seq, prompt, sizeof(int32_t) * n_prompt);
    int32_t len = n_prompt, model = ORACLE_SMALL, c = 0, n = 0, rc = 0;
    while (n < max_new) {
        /* l <- M_t(x + y): bring the active model's cache up to date */
        oracle_cache *cc = cache[model];
        while (cc->len < len) {
            int last = (cc->len == len - 1);
            if (oracle_forward_cached(mdl[model], cc, seq[cc->len], last ? logits : NULL)) { rc = -2; goto done; }
        }
        int32_t tok;
        float H = (float)oracle_entropy(logits, V, unit, &tok);      /* entropy of the raw logits */
        if (temperature > 0.0f) tok = oracle_sample(logits, V, temperature, seed, seq_index, n);
        W[n] = H;
        float Hbar = oracle_window_mean(W, n + 1, w);
        out_tokens[n] = tok; out_model[n] = (uint8_t)model; out_H[n] = H;
        if (out_Hbar) out_Hbar[n] = Hbar;
        seq[len++] = tok; ++n;
        oracle_gate_step(&model, &c, Hbar, tau, d_min);
        if (eos_id >= 0 && tok == eos_id) break;
    }
    rc = n;
done:
    oracle_cache_free(cache[0]); oracle_cache_free(cache[1]);
    free(seq); free(logits); free(W);
    return rc;
}

int32_t oracle_generate(const oracle_model *small, const oracle_model *large,
                        const int32_t *prompt, int32_t n_prompt, int32_t max_new,
                        int32_t w, float tau, int32_t d_min, int32_t unit, int32_t eos_id,
                        int32_t *out_tokens, uint8_t *out_model, float *out_H, float *out_Hbar)
{
    return oracle_generate_sampled(small, large, prompt, n_prompt, max_new, w, tau, d_min, unit, eos_id,
                                   0.0f, 0u, 0, out_tokens, out_model, out_H, out_Hbar);
}

int32_t oracle_num_threads(void)
{
    int32_t n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = (int32_t)omp_get_num_threads();
    }
#endif
    return n;
}
