// Small kernels both kernel families use: block set-up (embedding gather + rotary table),
// rotary embedding + KV append into pages, vocabulary argmax, the acceptance rule, KV export.
// None of them is bandwidth relevant; they are written for clarity and determinism.
#include "pv_kernels_common.h"

// ---------------------------------------------------------------------------------------
// Block set-up: x[j,:] = E[draft[j],:] and the rotary table of positions len .. len+gamma-1.
// Angles are formed in double (pos * base^(-2i/head_dim)) so that large positions lose no
// precision before sin/cos; the table is stored as float2 (cos, sin).
// ---------------------------------------------------------------------------------------
// The draft ids are read straight from the cache's pinned host mailbox; block 0 copies them, the
// row count and the mode into the device state for the kernels that follow.
template <typename ST>
__global__ void __launch_bounds__(256)
k_begin(pv_dev_state *st, const int32_t *mailbox, int gamma, int mode, const ST *embed, const double *inv_freq, float *x, float2 *rope, int d, int half)
{
    const int j = blockIdx.x;
    if (j == 0) {
        if ((int)threadIdx.x < gamma) st->draft[threadIdx.x] = mailbox[threadIdx.x];
        if (threadIdx.x == 0) { st->gamma = gamma; st->mode = mode; st->blk.seq[0].gamma = gamma; }
    }
    float *xr = x + (size_t)j * d;
    if (j >= gamma) {                        // padding rows: keep them finite
        for (int i = threadIdx.x; i < d; i += 256) xr[i] = 0.f;
        for (int i = threadIdx.x; i < half; i += 256) rope[(size_t)j * half + i] = make_float2(1.f, 0.f);
        return;
    }
    const ST *e = embed + (size_t)mailbox[j] * d;
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
    if (threadIdx.x == 0) st->pred[j] = (sv[0] == -INFINITY) ? -1 : si[0];     // no finite logit in the row: no arg-max (k_finish reports it)
}

// ---------------------------------------------------------------------------------------
// End of a step in one launch: vocabulary arg-max of every row from the per-strip candidates the
// LM-head epilogue left (matrix path; the vector path has st->pred already), the acceptance rule
// (Algorithm 1, verify branch: longest draft prefix that equals the stage's own greedy tokens,
// one correction token) and the in-step rollback (length, pending).  The two results and an
// error flag go straight to the cache's pinned host mailbox.
// One workgroup of 16 waves: a row is scanned by 16 / (rows rounded up to a power of two) waves
// (one wave takes up to four rows when there are more than 16), sixteen candidates per lane in
// flight; after the barrier one thread per sequence of the block applies the rule.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(1024)
k_finish(pv_dev_state *st, int32_t *result, const float *pv, const int32_t *pi, int strips, int gamma, int mode, int vocab)
{
    __shared__ float wv[16];
    __shared__ int wi[16];
    __shared__ int pred_s[PV_MAX_ROWS];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (pv != nullptr && mode != PV_MODE_PREFILL_MID) {
        int wpr = 16;                                 // waves per row
        while (wpr > 1 && gamma * wpr > 16) wpr >>= 1;
        for (int j0 = 0; j0 < gamma; j0 += 16 / wpr) {           // one pass unless there are more than 16 rows
            const int j = j0 + wave / wpr, part = wave % wpr;
            float bv = -INFINITY; int bi = 0x7fffffff;
            if (j < gamma) {
                const float *rv = pv + (size_t)j * strips; const int32_t *ri = pi + (size_t)j * strips;
                for (int s0 = part * 64 + lane; s0 < strips; s0 += 64 * wpr * 16) {
                    float v[16]; int i[16];
#pragma unroll
                    for (int u = 0; u < 16; ++u) { const int s = s0 + 64 * wpr * u, sc = s < strips ? s : s0; v[u] = rv[sc]; i[u] = ri[sc]; }
#pragma unroll
                    for (int u = 0; u < 16; ++u)
                        if (s0 + 64 * wpr * u < strips && pv_better(v[u], i[u], bv, bi)) { bv = v[u]; bi = i[u]; }
                }
            }
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
                if (pv_better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
            }
            if (lane == 0) { wv[wave] = bv; wi[wave] = bi; }
            __syncthreads();
            if ((int)threadIdx.x < 16 / wpr && j0 + (int)threadIdx.x < gamma) {
                float fv = wv[threadIdx.x * wpr]; int fi = wi[threadIdx.x * wpr];
                for (int w = 1; w < wpr; ++w) if (pv_better(wv[threadIdx.x * wpr + w], wi[threadIdx.x * wpr + w], fv, fi)) { fv = wv[threadIdx.x * wpr + w]; fi = wi[threadIdx.x * wpr + w]; }
                pred_s[j0 + threadIdx.x] = (fv == -INFINITY) ? -1 : fi;     // no finite logit in the row: no arg-max
            }
            __syncthreads();
        }
    } else {
        if ((int)threadIdx.x < gamma) pred_s[threadIdx.x] = st->pred[threadIdx.x];
        __syncthreads();
    }
    // the rule, one thread per sequence of the block (a plain step has one: the cache itself)
    __shared__ int err_s;
    if (threadIdx.x == 0) err_s = 0;
    __syncthreads();
    const int nseq = st->blk.n_seq;
    if ((int)threadIdx.x < nseq) {
        const pv_seq_ref sq = st->blk.seq[threadIdx.x];
        pv_dev_state *ps = sq.st;                    // the sequence's own state
        const int g = sq.gamma, r0 = sq.row0;
        int n, next, err = 0;
        if (mode == PV_MODE_PREFILL_MID) { n = g; next = -1; }
        else {
            // a row without a finite logit has no arg-max: the step reports an error and commits nothing
            for (int j = 0; j < g; ++j) { if (pred_s[r0 + j] < 0 || pred_s[r0 + j] >= vocab) err = 1; st->pred[r0 + j] = pred_s[r0 + j]; }
            if (err) { n = 0; next = ps->pending; }
            else if (mode == PV_MODE_PREFILL_LAST) { n = g; next = pred_s[r0 + g - 1]; }
            else if (mode == PV_MODE_TREE) {
                // Greedy walk down the draft tree: at every step the child (lowest row first) whose token is the one
                // the stage itself predicts next is taken; its own prediction is then what its children must match.
                // The rows of the path are left in st->path for the compaction of their keys and values.
                int cur = -1, expected = ps->pending;
                n = 0;
                for (;;) {
                    int pick = -1;
                    for (int r = cur + 1; r < g && pick < 0; ++r)
                        if (st->parent[r] == cur && (expected < 0 ? true : st->draft[r] == expected)) pick = r;     // (pending unknown: the first root is trusted)
                    if (pick < 0) break;
                    st->path[n++] = pick;
                    cur = pick; expected = pred_s[pick];
                }
                next = (n >= 1) ? pred_s[cur] : ps->pending;
            }
            else {
                n = 0;
                while (n < g) {
                    const int expected = (n == 0) ? (ps->pending >= 0 ? ps->pending : st->draft[r0]) : pred_s[r0 + n - 1];
                    if (st->draft[r0 + n] != expected) break;
                    ++n;
                }
                next = (n >= 1) ? pred_s[r0 + n - 1] : ps->pending;
            }
        }
        ps->accepted = n;
        ps->next_token = next;
        ps->pending = next;
        ps->len += n;
        result[2 * threadIdx.x] = n; result[2 * threadIdx.x + 1] = next;
        if (err) err_s = 1;
    }
    __syncthreads();
    if (threadIdx.x == 0) result[PV_RESULT_ERR] = err_s;
}

// ---------------------------------------------------------------------------------------
// After a draft-tree step: the accepted path's rows sit in the slots of their row numbers
// (old length + path[d]); move their keys and values to the positions they now hold
// (old length + d).  path[] is increasing and path[d] >= d, so going through d in order never
// overwrites a row that is still to be moved.  One thread per (layer, K|V, kv head, feature).
// ---------------------------------------------------------------------------------------
template <typename ST>
__global__ void __launch_bounds__(256)
k_tree_compact(const pv_dev_state *st, const int32_t *page_table, ST *pool, pv_kv_geom g, int n_layers)
{
    const int kvd = g.n_kv_heads * g.head_dim;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)n_layers * 2 * kvd) return;
    const int c = (int)(idx % kvd), which = (int)((idx / kvd) & 1), layer = (int)(idx / kvd / 2);
    const int h = c / g.head_dim, e = c - h * g.head_dim;
    const int n = st->accepted, len0 = st->len - n;          // (the finishing kernel has added n already)
    for (int d = 0; d < n; ++d) {
        const int src = len0 + st->path[d], dst = len0 + d;
        if (src == dst) continue;
        const ST *sb = pool + pv_kv_block(g, layer, page_table[src >> g.page_shift], h, which);
        ST *db = pool + pv_kv_block(g, layer, page_table[dst >> g.page_shift], h, which);
        const int ts = src & (g.page_tokens - 1), td = dst & (g.page_tokens - 1);
        db[which ? pv_v_off(g, td, e) : pv_k_off(g, td, e)] = sb[which ? pv_v_off(g, ts, e) : pv_k_off(g, ts, e)];
    }
}

__global__ void k_set_state(pv_dev_state *st, int len, int pending)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) { st->len = len; st->pending = pending; }
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
    const int rows = c->last_rows, mode = c->io->hdr[3];
    if (m->cfg.dtype == PV_BF16)
        k_begin<uint16_t><<<rows_pad, 256, 0, s>>>(c->ws.state, c->d_io->draft, rows, mode, (const uint16_t *)emb, inv, c->ws.x, c->ws.rope, m->cfg.d_model, m->cfg.head_dim / 2);
    else
        k_begin<float><<<rows_pad, 256, 0, s>>>(c->ws.state, c->d_io->draft, rows, mode, (const float *)emb, inv, c->ws.x, c->ws.rope, m->cfg.d_model, m->cfg.head_dim / 2);
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

int pv_k_argmax(pv_cache *c, int rows, hipStream_t s)
{
    k_argmax<<<rows, 1024, 0, s>>>(c->ws.state, c->ws.logits, c->m->cfg.vocab);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

// pmax_val / pmax_idx: per-strip arg-max candidates [rows][strips] (null: st->pred is already filled in)
int pv_k_finish(pv_cache *c, int rows, const float *pmax_val, const int32_t *pmax_idx, int strips, hipStream_t s)
{
    k_finish<<<1, 1024, 0, s>>>(c->ws.state, c->d_io->result, pmax_val, pmax_idx, strips, rows, c->io->hdr[3], c->m->cfg.vocab);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_tree_compact(pv_cache *c, hipStream_t s)
{
    const pv_kv_geom g = pv_geom(c);
    const size_t n = (size_t)c->m->cfg.n_layers * 2 * g.n_kv_heads * g.head_dim;
    const unsigned blocks = (unsigned)((n + 255) / 256);
    if (c->m->cfg.dtype == PV_BF16)
        k_tree_compact<uint16_t><<<blocks, 256, 0, s>>>(c->ws.state, c->ws.page_table, (uint16_t *)c->d_pool, g, c->m->cfg.n_layers);
    else
        k_tree_compact<float><<<blocks, 256, 0, s>>>(c->ws.state, c->ws.page_table, (float *)c->d_pool, g, c->m->cfg.n_layers);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

int pv_k_set_state(pv_cache *c, int len, int pending, hipStream_t s)
{
    k_set_state<<<1, 64, 0, s>>>(c->ws.state, len, pending);
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
