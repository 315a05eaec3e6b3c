/*
 * CPU oracle for the verification step of one PipeSpec pipeline stage.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may include, link or
 * call this file; it exists so that the GPU library can be checked against a
 * plain statement of what the step computes, and to be timed as the CPU
 * baseline.  It shares no code with the GPU path.
 *
 * What it computes (paper: Sec. 3.2, Algorithm 1, the "verify drafts" branch;
 * Sec. 3.3, the remark after Eq. 1 that a rejecting verifier emits one token of
 * its own; Sec. 4.1, greedy decoding at temperature 0):
 *   - a LLaMA-style decoder forward (RMSNorm, rotary embedding with the
 *     rotate-half pairing, causal grouped-query attention, SwiGLU, untied LM
 *     head) over tokens appended to a key/value cache,
 *   - per-position argmax (ties -> lowest id),
 *   - acceptance of the longest draft prefix that equals greedy decoding, plus
 *     one correction token, and truncation of the cache past the rejection.
 * The paper names the model family only; the layer equations are the public
 * LLaMA definition, written here in their textbook form.
 *
 * Arithmetic type: `real` (double unless -DPV_REAL=float).  Stored weights are
 * float32 or bfloat16 bit patterns, widened exactly.  K/V may be kept in
 * `real`, or rounded on store to the cache's storage type (bf16 / f32).
 *
 * Two independent forward routines: ref_decode_one (one token; loops over the
 * cached positions) and ref_forward_block (n rows at once; full score matrix
 * with an explicit mask).  Tests require them to agree.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifndef PV_REAL
#define PV_REAL double
#endif
typedef PV_REAL real;

enum { REF_F32 = 0, REF_BF16 = 1 };
enum { REF_KV_REAL = 0, REF_KV_BF16 = 1, REF_KV_F32 = 2 };
enum {
    T_EMBED = 0, T_ATTN_NORM, T_WQ, T_WK, T_WV, T_WO, T_FFN_NORM, T_WG, T_WU, T_WD,
    T_FINAL_NORM, T_LM_HEAD, T_NKINDS
};

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
    double rms_eps, rope_base;
} ref_config;

typedef struct { const void *data; int dtype; } ref_tensor;

typedef struct {
    ref_config c;
    ref_tensor *layer;               /* [n_layers][T_NKINDS] */
    ref_tensor global[T_NKINDS];
} ref_model;

typedef struct {
    const ref_model *m;
    int32_t max_tokens, len, kv_store;
    real *K, *V;                     /* [n_layers][max_tokens][n_kv_heads*head_dim] */
} ref_cache;

int ref_sizeof_real(void) { return (int)sizeof(real); }

/* ---------- element access ---------- */

static inline float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16; float f; memcpy(&f, &u, 4); return f;
}

static inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

static inline real store_round(real v, int mode)
{
    if (mode == REF_KV_BF16) return (real)bf16_to_f32(f32_to_bf16_rne((float)v));
    if (mode == REF_KV_F32) return (real)(float)v;
    return v;
}

/* the cache's store rounding on its own, so that tests can pin it against a library conversion */
real ref_store_round(real v, int mode) { return store_round(v, mode); }

static inline real tget(const ref_tensor *t, size_t i)
{
    return t->dtype == REF_BF16 ? (real)bf16_to_f32(((const uint16_t *)t->data)[i])
                                : (real)((const float *)t->data)[i];
}

/* dot(x[0..n), row `r` of W[., n]) */
static real dot_row(const real *x, const ref_tensor *W, size_t r, int n)
{
    real acc = 0;
    if (W->dtype == REF_BF16) {
        const uint16_t *w = (const uint16_t *)W->data + r * (size_t)n;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < n; ++k) acc += x[k] * (real)bf16_to_f32(w[k]);
    } else {
        const float *w = (const float *)W->data + r * (size_t)n;
#pragma omp simd reduction(+ : acc)
        for (int k = 0; k < n; ++k) acc += x[k] * (real)w[k];
    }
    return acc;
}

/* ---------- layer pieces (each exported so tests can pin it alone) ---------- */

/* y = x * rsqrt(mean(x^2) + eps) * g */
void ref_rmsnorm(const real *x, const ref_tensor *g, int d, double eps, real *y)
{
    real ss = 0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    real r = (real)1 / (real)sqrt((double)(ss / (real)d) + eps);
    for (int i = 0; i < d; ++i) y[i] = x[i] * r * tget(g, (size_t)i);
}

/* rows x [n_in] times W[n_out][n_in]^T -> y rows x [n_out] */
void ref_linear(const real *x, int rows, const ref_tensor *W, int n_out, int n_in, real *y)
{
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; ++o)
        for (int r = 0; r < rows; ++r)
            y[(size_t)r * n_out + o] = dot_row(x + (size_t)r * n_in, W, (size_t)o, n_in);
}

/* rotate-half rotary embedding of one head vector at absolute position pos */
void ref_rope(real *v, int head_dim, int pos, double base)
{
    int half = head_dim / 2;
    for (int i = 0; i < half; ++i) {
        double theta = pow(base, -2.0 * (double)i / (double)head_dim);
        double ang = (double)pos * theta;
        real c = (real)cos(ang), s = (real)sin(ang);
        real a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

real ref_silu(real z) { return z / ((real)1 + (real)exp(-(double)z)); }

static int argmax_first(const real *v, int n)
{
    int best = 0;
    for (int i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

/* ---------- model / cache ---------- */

ref_model *ref_model_new(const ref_config *c)
{
    ref_model *m = (ref_model *)calloc(1, sizeof(ref_model));
    m->c = *c;
    m->layer = (ref_tensor *)calloc((size_t)c->n_layers * T_NKINDS, sizeof(ref_tensor));
    return m;
}

void ref_model_free(ref_model *m) { if (m) { free(m->layer); free(m); } }

/* data is borrowed: the caller keeps it alive for the model's lifetime */
int ref_model_set_tensor(ref_model *m, int kind, int layer, const void *data, int dtype)
{
    if (kind < 0 || kind >= T_NKINDS) return -1;
    ref_tensor t = { data, dtype };
    if (kind == T_EMBED || kind == T_FINAL_NORM || kind == T_LM_HEAD) m->global[kind] = t;
    else { if (layer < 0 || layer >= m->c.n_layers) return -1; m->layer[(size_t)layer * T_NKINDS + kind] = t; }
    return 0;
}

static const ref_tensor *LT(const ref_model *m, int l, int kind) { return &m->layer[(size_t)l * T_NKINDS + kind]; }

ref_cache *ref_cache_new(const ref_model *m, int max_tokens, int kv_store)
{
    ref_cache *c = (ref_cache *)calloc(1, sizeof(ref_cache));
    size_t n = (size_t)m->c.n_layers * max_tokens * m->c.n_kv_heads * m->c.head_dim;
    c->m = m; c->max_tokens = max_tokens; c->kv_store = kv_store;
    c->K = (real *)calloc(n, sizeof(real));
    c->V = (real *)calloc(n, sizeof(real));
    return c;
}

void ref_cache_free(ref_cache *c) { if (c) { free(c->K); free(c->V); free(c); } }
int ref_cache_len(const ref_cache *c) { return c->len; }

int ref_truncate(ref_cache *c, int new_len)
{
    if (new_len < 0 || new_len > c->len) return -1;
    c->len = new_len;
    return 0;
}

static real *kv_at(const ref_cache *c, real *base, int l, int pos)
{
    size_t kvd = (size_t)c->m->c.n_kv_heads * c->m->c.head_dim;
    return base + ((size_t)l * c->max_tokens + pos) * kvd;
}

/* logical K/V of the first len positions: out[l][2][len][kv_dim] */
void ref_cache_export(const ref_cache *c, real *out)
{
    size_t kvd = (size_t)c->m->c.n_kv_heads * c->m->c.head_dim;
    for (int l = 0; l < c->m->c.n_layers; ++l)
        for (int w = 0; w < 2; ++w)
            for (int p = 0; p < c->len; ++p)
                memcpy(out + (((size_t)l * 2 + w) * c->len + p) * kvd,
                       kv_at(c, w ? c->V : c->K, l, p), kvd * sizeof(real));
}

/* ---------- forward, one token at a time ---------- */

/* Appends `token` at position c->len; writes the logits of that position (vocab reals). */
int ref_decode_one(ref_cache *c, int token, real *logits)
{
    const ref_config *g = &c->m->c;
    const int d = g->d_model, hd = g->head_dim, Hq = g->n_q_heads, Hkv = g->n_kv_heads;
    const int qd = Hq * hd, kvd = Hkv * hd, F = g->ffn_dim, pos = c->len, group = Hq / Hkv;
    if (pos >= c->max_tokens || token < 0 || token >= g->vocab) return -1;
    real *x = (real *)malloc(sizeof(real) * (size_t)(3 * d + 2 * qd + 2 * F + (pos + 1)));
    real *h = x + d, *q = h + d, *o = q + qd, *a = o + qd, *u = a + F, *xo = u + F, *w = xo + d;

    for (int i = 0; i < d; ++i) x[i] = tget(&c->m->global[T_EMBED], (size_t)token * d + i);
    for (int l = 0; l < g->n_layers; ++l) {
        real *kp = kv_at(c, c->K, l, pos), *vp = kv_at(c, c->V, l, pos);
        ref_rmsnorm(x, LT(c->m, l, T_ATTN_NORM), d, g->rms_eps, h);
        ref_linear(h, 1, LT(c->m, l, T_WQ), qd, d, q);
        ref_linear(h, 1, LT(c->m, l, T_WK), kvd, d, kp);
        ref_linear(h, 1, LT(c->m, l, T_WV), kvd, d, vp);
        for (int hq = 0; hq < Hq; ++hq) ref_rope(q + hq * hd, hd, pos, g->rope_base);
        for (int hk = 0; hk < Hkv; ++hk) ref_rope(kp + hk * hd, hd, pos, g->rope_base);
        for (int i = 0; i < kvd; ++i) { kp[i] = store_round(kp[i], c->kv_store); vp[i] = store_round(vp[i], c->kv_store); }

        const real scale = (real)1 / (real)sqrt((double)hd);
        for (int hq = 0; hq < Hq; ++hq) {
            const int hk = hq / group;
            const real *qh = q + hq * hd;
            real mx = -INFINITY;
            for (int p = 0; p <= pos; ++p) {
                const real *kh = kv_at(c, c->K, l, p) + hk * hd;
                real s = 0;
                for (int e = 0; e < hd; ++e) s += qh[e] * kh[e];
                w[p] = s * scale;
                if (w[p] > mx) mx = w[p];
            }
            real den = 0;
            for (int p = 0; p <= pos; ++p) { w[p] = (real)exp((double)(w[p] - mx)); den += w[p]; }
            real *oh = o + hq * hd;
            for (int e = 0; e < hd; ++e) oh[e] = 0;
            for (int p = 0; p <= pos; ++p) {
                const real *vh = kv_at(c, c->V, l, p) + hk * hd;
                const real wp = w[p] / den;
                for (int e = 0; e < hd; ++e) oh[e] += wp * vh[e];
            }
        }
        ref_linear(o, 1, LT(c->m, l, T_WO), d, qd, xo);
        for (int i = 0; i < d; ++i) x[i] += xo[i];

        ref_rmsnorm(x, LT(c->m, l, T_FFN_NORM), d, g->rms_eps, h);
        ref_linear(h, 1, LT(c->m, l, T_WG), F, d, a);
        ref_linear(h, 1, LT(c->m, l, T_WU), F, d, u);
        for (int i = 0; i < F; ++i) a[i] = ref_silu(a[i]) * u[i];
        ref_linear(a, 1, LT(c->m, l, T_WD), d, F, xo);
        for (int i = 0; i < d; ++i) x[i] += xo[i];
    }
    ref_rmsnorm(x, &c->m->global[T_FINAL_NORM], d, g->rms_eps, h);
    ref_linear(h, 1, &c->m->global[T_LM_HEAD], g->vocab, d, logits);
    c->len = pos + 1;
    free(x);
    return 0;
}

/* ---------- forward, a block of n rows at once ---------- */

/* X[j][:] = E[tokens[j]][:] */
int ref_embed_block(const ref_model *m, const int32_t *tokens, int n, real *X)
{
    const int d = m->c.d_model;
    for (int j = 0; j < n; ++j) if (tokens[j] < 0 || tokens[j] >= m->c.vocab) return -1;
    for (int j = 0; j < n; ++j)
        for (int i = 0; i < d; ++i) X[(size_t)j * d + i] = tget(&m->global[T_EMBED], (size_t)tokens[j] * d + i);
    return 0;
}

/*
 * Decoder layer l over the n rows X[n][d_model] (in place) that sit at positions
 * T .. T+n-1: their keys and values are written to the cache at those positions,
 * row j may attend to position p iff p <= T+j, expressed as an explicit
 * n x (T+n) 0/1 mask over the full score matrix.  Only layer l's tensors need to
 * be set in the model.  The cache length is not touched: a driver that goes
 * through a deep model layer by layer (one layer's weights alive at a time) calls
 * this for every block of rows of a layer before moving to the next layer.
 */
int ref_layer_block(ref_cache *c, int l, int T, real *X, int n)
{
    const ref_config *g = &c->m->c;
    const int d = g->d_model, hd = g->head_dim, Hq = g->n_q_heads, Hkv = g->n_kv_heads;
    const int qd = Hq * hd, kvd = Hkv * hd, F = g->ffn_dim, S = T + n, group = Hq / Hkv;
    if (n <= 0 || T < 0 || S > c->max_tokens || l < 0 || l >= g->n_layers) return -1;

    real *H = (real *)malloc(sizeof(real) * (size_t)n * (size_t)(2 * d + 2 * qd + 2 * F));
    real *XO = H + (size_t)n * d, *Q = XO + (size_t)n * d;
    real *O = Q + (size_t)n * qd, *A = O + (size_t)n * qd, *U = A + (size_t)n * F;
    unsigned char *mask = (unsigned char *)malloc((size_t)n * S);
    for (int j = 0; j < n; ++j) for (int p = 0; p < S; ++p) mask[(size_t)j * S + p] = (p <= T + j);

    real *Kl = kv_at(c, c->K, l, 0), *Vl = kv_at(c, c->V, l, 0);   /* [max_tokens][kvd] */
    for (int j = 0; j < n; ++j) ref_rmsnorm(X + (size_t)j * d, LT(c->m, l, T_ATTN_NORM), d, g->rms_eps, H + (size_t)j * d);
    ref_linear(H, n, LT(c->m, l, T_WQ), qd, d, Q);
    ref_linear(H, n, LT(c->m, l, T_WK), kvd, d, Kl + (size_t)T * kvd);
    ref_linear(H, n, LT(c->m, l, T_WV), kvd, d, Vl + (size_t)T * kvd);
    for (int j = 0; j < n; ++j) {
        for (int hq = 0; hq < Hq; ++hq) ref_rope(Q + (size_t)j * qd + hq * hd, hd, T + j, g->rope_base);
        for (int hk = 0; hk < Hkv; ++hk) ref_rope(Kl + (size_t)(T + j) * kvd + hk * hd, hd, T + j, g->rope_base);
        for (int i = 0; i < kvd; ++i) {
            real *kk = Kl + (size_t)(T + j) * kvd + i, *vv = Vl + (size_t)(T + j) * kvd + i;
            *kk = store_round(*kk, c->kv_store); *vv = store_round(*vv, c->kv_store);
        }
    }
    const real scale = (real)1 / (real)sqrt((double)hd);
#pragma omp parallel for schedule(static)
    for (int hq = 0; hq < Hq; ++hq) {
        const int hk = hq / group;
        real *P = (real *)malloc(sizeof(real) * (size_t)n * S);
        /* scores = Q_h K_h^T / sqrt(hd), masked entries -> -inf */
        for (int j = 0; j < n; ++j)
            for (int p = 0; p < S; ++p) {
                real s = 0;
                const real *qh = Q + (size_t)j * qd + hq * hd, *kh = Kl + (size_t)p * kvd + hk * hd;
                for (int e = 0; e < hd; ++e) s += qh[e] * kh[e];
                P[(size_t)j * S + p] = mask[(size_t)j * S + p] ? s * scale : -INFINITY;
            }
        /* row softmax */
        for (int j = 0; j < n; ++j) {
            real *row = P + (size_t)j * S, mx = -INFINITY, den = 0;
            for (int p = 0; p < S; ++p) if (row[p] > mx) mx = row[p];
            for (int p = 0; p < S; ++p) { row[p] = (real)exp((double)(row[p] - mx)); den += row[p]; }
            for (int p = 0; p < S; ++p) row[p] /= den;
        }
        /* O_h = P V_h */
        for (int j = 0; j < n; ++j) {
            real *oh = O + (size_t)j * qd + hq * hd;
            for (int e = 0; e < hd; ++e) oh[e] = 0;
            for (int p = 0; p < S; ++p) {
                const real wp = P[(size_t)j * S + p];
                const real *vh = Vl + (size_t)p * kvd + hk * hd;
                for (int e = 0; e < hd; ++e) oh[e] += wp * vh[e];
            }
        }
        free(P);
    }
    ref_linear(O, n, LT(c->m, l, T_WO), d, qd, XO);
    for (size_t i = 0; i < (size_t)n * d; ++i) X[i] += XO[i];

    for (int j = 0; j < n; ++j) ref_rmsnorm(X + (size_t)j * d, LT(c->m, l, T_FFN_NORM), d, g->rms_eps, H + (size_t)j * d);
    ref_linear(H, n, LT(c->m, l, T_WG), F, d, A);
    ref_linear(H, n, LT(c->m, l, T_WU), F, d, U);
    for (size_t i = 0; i < (size_t)n * F; ++i) A[i] = ref_silu(A[i]) * U[i];
    ref_linear(A, n, LT(c->m, l, T_WD), d, F, XO);
    for (size_t i = 0; i < (size_t)n * d; ++i) X[i] += XO[i];
    free(mask); free(H);
    return 0;
}

/* logits[j][:] = rmsnorm(X[j]; g_final) W_out^T for the n rows of X */
int ref_head_block(const ref_model *m, const real *X, int n, real *logits)
{
    const int d = m->c.d_model;
    real *H = (real *)malloc(sizeof(real) * (size_t)n * d);
    for (int j = 0; j < n; ++j) ref_rmsnorm(X + (size_t)j * d, &m->global[T_FINAL_NORM], d, m->c.rms_eps, H + (size_t)j * d);
    ref_linear(H, n, &m->global[T_LM_HEAD], m->c.vocab, d, logits);
    free(H);
    return 0;
}

/* set the committed length directly (a layer-by-layer driver commits after the last layer) */
int ref_cache_set_len(ref_cache *c, int len)
{
    if (len < 0 || len > c->max_tokens) return -1;
    c->len = len;
    return 0;
}

/*
 * Appends tokens[0..n) at positions len..len+n-1.  logits (nullable) receives
 * [n][vocab]; if only_last != 0 just the last row's logits are computed and
 * written to logits[0..vocab).
 */
int ref_forward_block(ref_cache *c, const int32_t *tokens, int n, real *logits, int only_last)
{
    const ref_config *g = &c->m->c;
    const int d = g->d_model, T = c->len, S = T + n;
    if (n <= 0 || S > c->max_tokens) return -1;
    real *X = (real *)malloc(sizeof(real) * (size_t)n * d);
    if (ref_embed_block(c->m, tokens, n, X) != 0) { free(X); return -1; }
    for (int l = 0; l < g->n_layers; ++l) ref_layer_block(c, l, T, X, n);
    if (logits) {
        int j0 = only_last ? n - 1 : 0;
        ref_head_block(c->m, X + (size_t)j0 * d, n - j0, logits);
    }
    c->len = S;
    free(X);
    return 0;
}

/* ---------- the verification step ---------- */

/*
 * Verify draft[0..gamma) on top of the cached prefix (Algorithm 1, verify branch).
 *   pred[j]     = argmax of the logits after consuming draft[0..j]
 *   expected[0] = *pending if known (>= 0), else draft[0] is trusted
 *   expected[j] = pred[j-1]
 *   n           = length of the longest prefix with draft[j] == expected[j]
 *   next_token  = pred[n-1] if n >= 1 else *pending
 * Afterwards the cache holds prefix + draft[0..n) and *pending = next_token.
 * pred_out (nullable, gamma ints) and logits (nullable, [gamma][vocab]) expose
 * the intermediate results.  Returns 0, or -1 on a bad argument / state.
 */
int ref_verify(ref_cache *c, int prefix_len, const int32_t *draft, int gamma, int32_t *pending,
               int32_t *accepted_len, int32_t *next_token, int32_t *pred_out, real *logits)
{
    const int V = c->m->c.vocab;
    if (prefix_len != c->len || gamma <= 0) return -1;
    real *lg = logits ? logits : (real *)malloc(sizeof(real) * (size_t)gamma * V);
    if (ref_forward_block(c, draft, gamma, lg, 0) != 0) { if (!logits) free(lg); return -1; }
    int32_t *pred = (int32_t *)malloc(sizeof(int32_t) * gamma);
    for (int j = 0; j < gamma; ++j) pred[j] = argmax_first(lg + (size_t)j * V, V);
    int n = 0;
    while (n < gamma) {
        int32_t expected = (n == 0) ? (*pending >= 0 ? *pending : draft[0]) : pred[n - 1];
        if (draft[n] != expected) break;
        ++n;
    }
    *accepted_len = n;
    *next_token = (n >= 1) ? pred[n - 1] : *pending;
    *pending = *next_token;
    ref_truncate(c, prefix_len + n);
    if (pred_out) memcpy(pred_out, pred, sizeof(int32_t) * gamma);
    free(pred);
    if (!logits) free(lg);
    return 0;
}
