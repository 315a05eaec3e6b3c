// Small kernels both kernel families use: block set-up (embedding gather + rotary table),
// rotary embedding + KV append into pages, vocabulary argmax, the acceptance rule, KV export.
// None of them is bandwidth relevant; they are written for clarity and determinism.
#include "pv_kernels_common.h"

// ---------------------------------------------------------------------------------------
// Block set-up: x[j,:] = E[draft[j],:] and the rotary table of positions len .. len+gamma-1.
// Angles are formed in double (pos * base^(-2i/head_dim)) so that large positions lose no
// precision before sin/cos; the table is stored as float2 (cos, sin).
// ---------------------------------------------------------------------------------------
template <typename ST>
__global__ void __launch_bounds__(256)
k_begin(const pv_dev_state *st, const ST *embed, const double *inv_freq, float *x, float2 *rope, int d, int half)
{
    const int j = blockIdx.x, gamma = st->gamma;
    float *xr = x + (size_t)j * d;
    if (j >= gamma) {                        // padding rows: keep them finite
        for (int i = threadIdx.x; i < d; i += 256) xr[i] = 0.f;
        for (int i = threadIdx.x; i < half; i += 256) rope[(size_t)j * half + i] = make_float2(1.f, 0.f);
        return;
    }
    const ST *e = embed + (size_t)st->draft[j] * d;
    for (int i = threadIdx.x; i < d; i += 256) xr[i] = pv_ld(e, i);
    const double pos = (double)(st->len + j);
    for (int i = threadIdx.x; i < half; i += 256) {
        double s, c;
        sincos(pos * inv_freq[i], &s, &c);
        rope[(size_t)j * half + i] = make_float2((float)c, (float)s);
    }
}

// ---------------------------------------------------------------------------------------
// Rotary embedding of q (in place) and k, then append k and v of row j at position len+j.
// K page block is [token][head_dim]; V page block is [head_dim][token].
// ---------------------------------------------------------------------------------------
template <typename ST>
__global__ void __launch_bounds__(256)
k_rope_append(const pv_dev_state *st, const int32_t *page_table, const float2 *rope, float *q,
              const float *k, const float *v, ST *pool, pv_kv_geom g, int layer, int n_q_heads)
{
    const int j = blockIdx.x;
    if (j >= st->gamma) return;
    const int hd = g.head_dim, half = hd / 2;
    const float2 *cs = rope + (size_t)j * half;
    float *qr = q + (size_t)j * n_q_heads * hd;
    for (int idx = threadIdx.x; idx < n_q_heads * half; idx += 256) {
        const int h = idx / half, i = idx - h * half;
        const float2 c = cs[i];
        const float a = qr[h * hd + i], b = qr[h * hd + i + half];
        qr[h * hd + i] = a * c.x - b * c.y;
        qr[h * hd + i + half] = b * c.x + a * c.y;
    }
    const int pos = st->len + j;
    const int phys = page_table[pos >> g.page_shift], tok = pos & (g.page_tokens - 1);
    const float *kr = k + (size_t)j * g.n_kv_heads * hd, *vr = v + (size_t)j * g.n_kv_heads * hd;
    for (int idx = threadIdx.x; idx < g.n_kv_heads * half; idx += 256) {
        const int h = idx / half, i = idx - h * half;
        const float2 c = cs[i];
        const float a = kr[h * hd + i], b = kr[h * hd + i + half];
        ST *kb = pool + pv_kv_block(g, layer, phys, h, 0);
        pv_st(kb, pv_k_off(g, tok, i), a * c.x - b * c.y);
        pv_st(kb, pv_k_off(g, tok, i + half), b * c.x + a * c.y);
    }
    for (int idx = threadIdx.x; idx < g.n_kv_heads * hd; idx += 256) {
        const int h = idx / hd, e = idx - h * hd;
        ST *vb = pool + pv_kv_block(g, layer, phys, h, 1);
        pv_st(vb, pv_v_off(g, tok, e), vr[h * hd + e]);
    }
}

// ---------------------------------------------------------------------------------------
// Row argmax over the vocabulary: order (value descending, index ascending); NaN counts as -inf.
// ---------------------------------------------------------------------------------------
__device__ inline bool pv_better(float v, int i, float bv, int bi) { return v > bv || (v == bv && i < bi); }

__global__ void __launch_bounds__(1024)
k_argmax(pv_dev_state *st, const float *logits, int vocab)
{
    const int j = blockIdx.x;
    if (j >= st->gamma) return;
    const float *row = logits + (size_t)j * vocab;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int i = threadIdx.x; i < vocab; i += 1024) {
        float v = row[i];
        v = (v == v) ? v : -INFINITY;
        if (pv_better(v, i, bv, bi)) { bv = v; bi = i; }
    }
    __shared__ float sv[1024];
    __shared__ int si[1024];
    sv[threadIdx.x] = bv; si[threadIdx.x] = bi;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if (threadIdx.x < s && pv_better(sv[threadIdx.x + s], si[threadIdx.x + s], sv[threadIdx.x], si[threadIdx.x])) {
            sv[threadIdx.x] = sv[threadIdx.x + s]; si[threadIdx.x] = si[threadIdx.x + s];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) st->pred[j] = si[0];
}

// ---------------------------------------------------------------------------------------
// Acceptance rule + in-step rollback (metadata).  One thread.
// ---------------------------------------------------------------------------------------
__global__ void k_accept(pv_dev_state *st)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    const int gamma = st->gamma;
    int n, next;
    if (st->mode == PV_MODE_PREFILL_MID) { n = gamma; next = -1; }
    else if (st->mode == PV_MODE_PREFILL_LAST) { n = gamma; next = st->pred[gamma - 1]; }
    else {
        n = 0;
        while (n < gamma) {
            const int expected = (n == 0) ? (st->pending >= 0 ? st->pending : st->draft[0]) : st->pred[n - 1];
            if (st->draft[n] != expected) break;
            ++n;
        }
        next = (n >= 1) ? st->pred[n - 1] : st->pending;
    }
    st->accepted = n;
    st->next_token = next;
    st->pending = next;
    st->len += n;
}

__global__ void k_set_state(pv_dev_state *st, int len, int pending)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { st->len = len; st->pending = pending; }
}

__global__ void k_set_step(pv_dev_state *st, int gamma, int mode)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { st->gamma = gamma; st->mode = mode; }
}

// ---------------------------------------------------------------------------------------
// Gather logical K/V elements [e0, e0+n) of the layout [layer][2][len][kv_dim] into out.
// ---------------------------------------------------------------------------------------
template <typename ST>
__global__ void k_export(const ST *pool, const int32_t *page_table, pv_kv_geom g, int len, size_t e0, size_t n, ST *out)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const size_t e = e0 + i;
    const int kvd = g.n_kv_heads * g.head_dim;
    const int c = (int)(e % kvd);
    const size_t r = e / kvd;
    const int pos = (int)(r % len);
    const size_t lw = r / len;
    const int which = (int)(lw & 1), layer = (int)(lw >> 1);
    const int h = c / g.head_dim, d = c - h * g.head_dim;
    const int phys = page_table[pos >> g.page_shift], tok = pos & (g.page_tokens - 1);
    const ST *b = pool + pv_kv_block(g, layer, phys, h, which);
    out[i] = which ? b[pv_v_off(g, tok, d)] : b[pv_k_off(g, tok, d)];
}

// ------------------------------- host launchers ----------------------------------------

pv_kv_geom pv_geom(const pv_cache *c)
{
    pv_kv_geom g;
    g.n_pages = c->n_pages; g.n_kv_heads = c->m->cfg.n_kv_heads; g.page_tokens = c->m->cfg.page_tokens;
    g.head_dim = c->m->cfg.head_dim;
    g.tiled = c->m->path >= PV_PATH_MATRIX;
    g.page_shift = 0;
    while ((1 << g.page_shift) < g.page_tokens) ++g.page_shift;
    return g;
}

int pv_k_begin(pv_cache *c, int rows_pad, hipStream_t s)
{
    const pv_model *m = c->m;
    const double *inv = (const double *)(m->d_weights + m->inv_freq_off);
    const void *emb = m->d_weights + m->global[PV_T_EMBED].off;
    if (m->cfg.dtype == PV_BF16)
        k_begin<uint16_t><<<rows_pad, 256, 0, s>>>(c->ws.state, (const uint16_t *)emb, inv, c->ws.x, c->ws.rope, m->cfg.d_model, m->cfg.head_dim / 2);
    else
        k_begin<float><<<rows_pad, 256, 0, s>>>(c->ws.state, (const float *)emb, inv, c->ws.x, c->ws.rope, m->cfg.d_model, m->cfg.head_dim / 2);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_rope_append(pv_cache *c, int layer, int rows, hipStream_t s)
{
    const pv_model *m = c->m;
    const pv_kv_geom g = pv_geom(c);
    if (m->cfg.dtype == PV_BF16)
        k_rope_append<uint16_t><<<rows, 256, 0, s>>>(c->ws.state, c->ws.page_table, c->ws.rope, c->ws.q, c->ws.k, c->ws.v,
                                                      (uint16_t *)c->d_pool, g, layer, m->cfg.n_q_heads);
    else
        k_rope_append<float><<<rows, 256, 0, s>>>(c->ws.state, c->ws.page_table, c->ws.rope, c->ws.q, c->ws.k, c->ws.v,
                                                   (float *)c->d_pool, g, layer, m->cfg.n_q_heads);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_argmax_accept(pv_cache *c, int rows, bool with_argmax, hipStream_t s)
{
    if (with_argmax) {
        k_argmax<<<rows, 1024, 0, s>>>(c->ws.state, c->ws.logits, c->m->cfg.vocab);
        PV_HIP(hipGetLastError());
    }
    k_accept<<<1, 64, 0, s>>>(c->ws.state);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_set_state(pv_cache *c, int len, int pending, hipStream_t s)
{
    k_set_state<<<1, 64, 0, s>>>(c->ws.state, len, pending);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_set_step(pv_cache *c, int gamma, int mode, hipStream_t s)
{
    k_set_step<<<1, 64, 0, s>>>(c->ws.state, gamma, mode);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_export(pv_cache *c, size_t e0, size_t n, void *d_out, hipStream_t s)
{
    const pv_kv_geom g = pv_geom(c);
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (c->m->cfg.dtype == PV_BF16)
        k_export<uint16_t><<<blocks, 256, 0, s>>>((const uint16_t *)c->d_pool, c->ws.page_table, g, c->len, e0, n, (uint16_t *)d_out);
    else
        k_export<float><<<blocks, 256, 0, s>>>((const float *)c->d_pool, c->ws.page_table, g, c->len, e0, n, (float *)d_out);
    PV_HIP(hipGetLastError());
    return PV_OK;
}
