// Host side of the C ABI declared in include/pipeverify.h: argument checks, arena / workspace
// layout, the per-step launch sequence, host mirrors of the cache state.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <stddef.h>
#include <new>
#include <mutex>
#include "pv_kernels_common.h"

static thread_local char g_err[512] = "";

void pv_set_error(const char *fmt, ...)
{
    va_list ap; va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char *pv_last_error(void) { return g_err; }

extern "C" const char *pv_strerror(int status)
{
    switch (status) {
    case PV_OK: return "ok";
    case PV_EINVAL: return "invalid argument";
    case PV_ESTATE: return "call not valid in the current state";
    case PV_ERANGE: return "value out of range";
    case PV_EHIP: return "HIP runtime error";
    case PV_ENOMEM: return "buffer too small";
    case PV_ENUMERIC: return "non-finite logits";
    default: return "unknown status";
    }
}

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline bool is_pow2(int v) { return v > 0 && (v & (v - 1)) == 0; }
static const size_t STAGING_BYTES = 64u << 20;

static int resolve_path(const pv_model_config *c)
{
    if (c->kernel_path == PV_PATH_AUTO) return c->dtype == PV_BF16 ? PV_PATH_MATRIX : PV_PATH_VECTOR;
    return c->kernel_path;
}

static int check_config(const pv_model_config *c)
{
    if (!c) { pv_set_error("null config"); return PV_EINVAL; }
    if (c->n_layers <= 0 || c->d_model <= 0 || c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->head_dim <= 0 ||
        c->ffn_dim <= 0 || c->vocab <= 0) { pv_set_error("non-positive dimension"); return PV_EINVAL; }
    if (c->n_q_heads % c->n_kv_heads) { pv_set_error("n_q_heads must be a multiple of n_kv_heads"); return PV_EINVAL; }
    if (c->head_dim % 2 || c->head_dim > 256) { pv_set_error("head_dim must be even and <= 256"); return PV_EINVAL; }
    if (c->dtype != PV_F32 && c->dtype != PV_BF16) { pv_set_error("bad dtype"); return PV_EINVAL; }
    if (!is_pow2(c->page_tokens)) { pv_set_error("page_tokens must be a power of two"); return PV_EINVAL; }
    if (c->max_gamma < 1 || c->max_gamma > PV_MAX_ROWS) { pv_set_error("max_gamma must be in [1, %d]", PV_MAX_ROWS); return PV_EINVAL; }
    if (!(c->rms_eps > 0) || !(c->rope_base > 1)) { pv_set_error("bad rms_eps / rope_base"); return PV_EINVAL; }
    const int path = resolve_path(c);
    if (path != PV_PATH_VECTOR && path != PV_PATH_MATRIX) { pv_set_error("bad kernel_path"); return PV_EINVAL; }
    const int qd = c->n_q_heads * c->head_dim;
    if (c->d_model % 4 || c->ffn_dim % 4 || qd % 4) { pv_set_error("d_model, ffn_dim, q_dim must be multiples of 4"); return PV_EINVAL; }
    if (c->weight_bits != 0 && c->weight_bits != 16 && c->weight_bits != 4) { pv_set_error("weight_bits must be 0, 16 or 4"); return PV_EINVAL; }
    if (c->weight_bits == 4) {
        if (path < PV_PATH_MATRIX || c->dtype != PV_BF16) { pv_set_error("4-bit weights need bf16 storage and the matrix path"); return PV_EINVAL; }
        if (c->d_model % 128 || c->ffn_dim % 128 || qd % 128) { pv_set_error("4-bit weights: d_model, ffn_dim, q_dim must be multiples of 128"); return PV_EINVAL; }
    }
    if (path >= PV_PATH_MATRIX) {
        if (c->dtype != PV_BF16) { pv_set_error("matrix path needs bf16 storage"); return PV_EINVAL; }
        if (c->d_model % 32 || c->ffn_dim % 32 || qd % 32 || c->vocab % 16 || (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128) || c->page_tokens < 16) {
            pv_set_error("matrix path: d_model, ffn_dim, q_dim %% 32, vocab %% 16, head_dim in {32, 64, 128}, page_tokens >= 16 required");
            return PV_EINVAL;
        }
    }
    return PV_OK;
}

static void tensor_dims(const pv_model_config *c, int kind, int64_t *rows, int64_t *cols)
{
    const int64_t d = c->d_model, qd = (int64_t)c->n_q_heads * c->head_dim, kvd = (int64_t)c->n_kv_heads * c->head_dim;
    switch (kind) {
    case PV_T_EMBED: case PV_T_LM_HEAD: *rows = c->vocab; *cols = d; break;
    case PV_T_ATTN_NORM: case PV_T_FFN_NORM: case PV_T_FINAL_NORM: *rows = 1; *cols = d; break;
    case PV_T_WQ: *rows = qd; *cols = d; break;
    case PV_T_WK: case PV_T_WV: *rows = kvd; *cols = d; break;
    case PV_T_WO: *rows = d; *cols = qd; break;
    case PV_T_WG: case PV_T_WU: *rows = c->ffn_dim; *cols = d; break;
    case PV_T_WD: *rows = d; *cols = c->ffn_dim; break;
    default: *rows = *cols = 0;
    }
}

// Lays the arena out; fills refs when m != nullptr.  Returns total bytes.
static size_t layout_arena(const pv_model_config *c, pv_model *m)
{
    const int path = resolve_path(c);
    const size_t elt = c->dtype == PV_BF16 ? 2 : 4;
    size_t off = 0;
    auto place = [&](int kind, int layer) {
        int64_t r, k; tensor_dims(c, kind, &r, &k);
        pv_tensor_ref t; t.off = off; t.rows = r; t.cols = k; t.loaded_rows = 0; t.strip_mul = 1; t.strip_add = 0;
        const size_t bytes = (c->weight_bits == 4 && pv_is_q4_kind(kind)) ? (size_t)(r / 16) * (k / 128) * PV_Q4_BATCH : (size_t)r * k * elt;
        off = align_up(off + bytes, 256);
        if (m) { if (layer < 0) m->global[kind] = t; else m->layer[(size_t)layer * PV_T_NKINDS + kind] = t; }
    };
    place(PV_T_EMBED, -1);
    for (int l = 0; l < c->n_layers; ++l) {
        place(PV_T_ATTN_NORM, l);
        place(PV_T_WQ, l); place(PV_T_WK, l); place(PV_T_WV, l);     // contiguous: one fused QKV region
        place(PV_T_WO, l);
        place(PV_T_FFN_NORM, l);
        const size_t gu = off;
        place(PV_T_WG, l); place(PV_T_WU, l);
        if (m && path >= PV_PATH_MATRIX) {                            // gate/up strips interleaved in one region
            pv_tensor_ref &g = m->layer[(size_t)l * PV_T_NKINDS + PV_T_WG], &u = m->layer[(size_t)l * PV_T_NKINDS + PV_T_WU];
            g.off = u.off = gu; g.strip_mul = u.strip_mul = 2; g.strip_add = 0; u.strip_add = 1;
        }
        place(PV_T_WD, l);
    }
    place(PV_T_FINAL_NORM, -1);
    place(PV_T_LM_HEAD, -1);
    if (m) m->inv_freq_off = off;
    off = align_up(off + (size_t)(c->head_dim / 2) * sizeof(double), 256);
    return off;
}

extern "C" int pv_model_bytes(const pv_model_config *cfg, size_t *weight_bytes, size_t *staging_bytes)
{
    int rc = check_config(cfg);
    if (rc != PV_OK) return rc;
    if (!weight_bytes || !staging_bytes) { pv_set_error("null output pointer"); return PV_EINVAL; }
    *weight_bytes = layout_arena(cfg, nullptr);
    *staging_bytes = resolve_path(cfg) >= PV_PATH_MATRIX ? STAGING_BYTES : 256;
    return PV_OK;
}

extern "C" int pv_model_create(const pv_model_config *cfg, void *d_weights, size_t weight_bytes,
                               void *d_staging, size_t staging_bytes, pv_model **out)
{
    int rc = check_config(cfg);
    if (rc != PV_OK) return rc;
    if (!d_weights || !d_staging || !out) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (((uintptr_t)d_weights | (uintptr_t)d_staging) & 255) { pv_set_error("device buffers must be 256-byte aligned"); return PV_EINVAL; }
    size_t need_w, need_s;
    pv_model_bytes(cfg, &need_w, &need_s);
    if (weight_bytes < need_w || staging_bytes < need_s) { pv_set_error("arena %zu < %zu or staging %zu < %zu", weight_bytes, need_w, staging_bytes, need_s); return PV_ENOMEM; }
    pv_model *m = new (std::nothrow) pv_model();
    if (!m) return PV_ENOMEM;
    m->cfg = *cfg; m->path = resolve_path(cfg); m->elt = cfg->dtype == PV_BF16 ? 2 : 4;
    m->wbits = cfg->weight_bits == 4 ? 4 : 16;
    m->d_weights = (char *)d_weights; m->weight_bytes = weight_bytes;
    m->d_staging = (char *)d_staging; m->staging_bytes = staging_bytes;
    m->layer = (pv_tensor_ref *)calloc((size_t)cfg->n_layers * PV_T_NKINDS, sizeof(pv_tensor_ref));
    if (!m->layer) { delete m; return PV_ENOMEM; }
    layout_arena(cfg, m);
    int dev = 0; hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        pv_set_error("no HIP device"); free(m->layer); delete m; return PV_EHIP;
    }
    m->n_cus = prop.multiProcessorCount;
    // rotary inverse frequencies base^(-2i/head_dim), double
    const int half = cfg->head_dim / 2;
    double *inv = (double *)malloc(sizeof(double) * half);
    for (int i = 0; i < half; ++i) inv[i] = pow(cfg->rope_base, -2.0 * (double)i / (double)cfg->head_dim);
    hipError_t e = hipMemcpy(m->d_weights + m->inv_freq_off, inv, sizeof(double) * half, hipMemcpyHostToDevice);
    free(inv);
    if (e != hipSuccess) { pv_set_error("upload of rotary table failed: %s", hipGetErrorString(e)); free(m->layer); delete m; return PV_EHIP; }
    *out = m;
    return PV_OK;
}

extern "C" void pv_model_destroy(pv_model *m)
{
    if (!m) return;
    free(m->layer);
    delete m;
}

// The rows of a tensor arrive in order: a chunk continues where the last one ended, or starts the
// tensor over at row 0.  (A row count alone would let overlapping chunks pass for a complete tensor.)
static int chunk_in_order(const pv_tensor_ref &t, int64_t row_begin)
{
    if (row_begin == 0 || row_begin == t.loaded_rows) return PV_OK;
    pv_set_error("rows of a tensor must be loaded in order: expected row_begin %lld (or 0 to start over), got %lld", (long long)t.loaded_rows, (long long)row_begin);
    return PV_ESTATE;
}

extern "C" int pv_load_weights(pv_model *m, int32_t kind, int32_t layer, int64_t row_begin, int64_t row_count,
                               const void *host_rows, void *hip_stream)
{
    if (!m || !host_rows) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (kind < 0 || kind >= PV_T_NKINDS) { pv_set_error("bad tensor kind %d", kind); return PV_EINVAL; }
    const bool global = kind == PV_T_EMBED || kind == PV_T_FINAL_NORM || kind == PV_T_LM_HEAD;
    if (!global && (layer < 0 || layer >= m->cfg.n_layers)) { pv_set_error("bad layer %d", layer); return PV_EINVAL; }
    pv_tensor_ref &t = global ? m->global[kind] : m->layer[(size_t)layer * PV_T_NKINDS + kind];
    if (row_begin < 0 || row_count <= 0 || row_begin + row_count > t.rows) { pv_set_error("rows [%lld, +%lld) outside tensor of %lld rows", (long long)row_begin, (long long)row_count, (long long)t.rows); return PV_ERANGE; }
    if (m->wbits == 4 && pv_is_q4_kind(kind)) { pv_set_error("tensor kind %d of a 4-bit model is loaded with pv_load_weights_q4", kind); return PV_EINVAL; }
    int orc = chunk_in_order(t, row_begin);
    if (orc != PV_OK) return orc;
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t nbytes = (size_t)row_count * t.cols * m->elt;
    const bool tiled = m->path >= PV_PATH_MATRIX && t.rows > 1 && kind != PV_T_EMBED;
    if (!tiled) {
        PV_HIP(hipMemcpyAsync(m->d_weights + t.off + (size_t)row_begin * t.cols * m->elt, host_rows, nbytes, hipMemcpyHostToDevice, s));
        PV_HIP(hipStreamSynchronize(s));
    } else {
        if ((row_begin | row_count) & 15) { pv_set_error("matrix path: row_begin and row_count must be multiples of 16"); return PV_EINVAL; }
        if (nbytes > m->staging_bytes) { pv_set_error("chunk of %zu bytes exceeds staging buffer of %zu", nbytes, m->staging_bytes); return PV_ENOMEM; }
        PV_HIP(hipMemcpyAsync(m->d_staging, host_rows, nbytes, hipMemcpyHostToDevice, s));
        int rc = pv_mat_repack(m, t, kind, row_begin, row_count, s);
        if (rc != PV_OK) return rc;
        PV_HIP(hipStreamSynchronize(s));
    }
    t.loaded_rows = row_begin + row_count;
    return PV_OK;
}

extern "C" int pv_load_weights_q4(pv_model *m, int32_t kind, int32_t layer, int64_t row_begin, int64_t row_count,
                                  const void *host_codes, const void *host_scales, void *hip_stream)
{
    if (!m || !host_codes || !host_scales) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (m->wbits != 4) { pv_set_error("not a 4-bit model"); return PV_ESTATE; }
    if (kind < 0 || kind >= PV_T_NKINDS || !pv_is_q4_kind(kind)) { pv_set_error("tensor kind %d is not stored in 4 bit", kind); return PV_EINVAL; }
    const bool global = kind == PV_T_LM_HEAD;
    if (!global && (layer < 0 || layer >= m->cfg.n_layers)) { pv_set_error("bad layer %d", layer); return PV_EINVAL; }
    pv_tensor_ref &t = global ? m->global[kind] : m->layer[(size_t)layer * PV_T_NKINDS + kind];
    if (row_begin < 0 || row_count <= 0 || row_begin + row_count > t.rows) { pv_set_error("rows [%lld, +%lld) outside tensor of %lld rows", (long long)row_begin, (long long)row_count, (long long)t.rows); return PV_ERANGE; }
    if ((row_begin | row_count) & 15) { pv_set_error("matrix path: row_begin and row_count must be multiples of 16"); return PV_EINVAL; }
    int orc = chunk_in_order(t, row_begin);
    if (orc != PV_OK) return orc;
    const size_t cbytes = (size_t)row_count * (t.cols / 2), sbytes = (size_t)row_count * (t.cols / PV_Q4_GROUP) * 2;
    const size_t soff = align_up(cbytes, 256);
    if (soff + sbytes > m->staging_bytes) { pv_set_error("chunk of %zu bytes exceeds staging buffer of %zu", soff + sbytes, m->staging_bytes); return PV_ENOMEM; }
    hipStream_t s = (hipStream_t)hip_stream;
    PV_HIP(hipMemcpyAsync(m->d_staging, host_codes, cbytes, hipMemcpyHostToDevice, s));
    PV_HIP(hipMemcpyAsync(m->d_staging + soff, host_scales, sbytes, hipMemcpyHostToDevice, s));
    int rc = pv_mat_repack_q4(m, t, kind, row_begin, row_count, soff, s);
    if (rc != PV_OK) return rc;
    PV_HIP(hipStreamSynchronize(s));
    t.loaded_rows = row_begin + row_count;
    return PV_OK;
}

static int model_complete(const pv_model *m)
{
    for (int k = 0; k < PV_T_NKINDS; ++k) {
        const bool global = k == PV_T_EMBED || k == PV_T_FINAL_NORM || k == PV_T_LM_HEAD;
        if (global) { if (m->global[k].loaded_rows < m->global[k].rows) return 0; }
        else for (int l = 0; l < m->cfg.n_layers; ++l) {
            const pv_tensor_ref &t = m->layer[(size_t)l * PV_T_NKINDS + k];
            if (t.loaded_rows < t.rows) return 0;
        }
    }
    return 1;
}

// ---- workspace layout ----
static size_t layout_ws(const pv_model *m, int rows_cap, int units_cap, int n_pages, pv_ws *w, char *base)
{
    const pv_model_config &c = m->cfg;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return base ? base + o : (char *)nullptr; };
    const size_t qd = (size_t)c.n_q_heads * c.head_dim, kvd = (size_t)c.n_kv_heads * c.head_dim, R = rows_cap;
    char *p;
    p = take(sizeof(pv_dev_state)); if (w) w->state = (pv_dev_state *)p;
    p = take(sizeof(int32_t) * n_pages); if (w) w->page_table = (int32_t *)p;
    p = take(sizeof(float2) * R * (c.head_dim / 2)); if (w) w->rope = (float2 *)p;
    p = take(4 * R * c.d_model); if (w) w->x = (float *)p;
    p = take(4 * R * c.d_model); if (w) w->h = (float *)p;
    p = take(4 * R * qd); if (w) w->q = (float *)p;
    p = take(4 * R * kvd); if (w) w->k = (float *)p;
    p = take(4 * R * kvd); if (w) w->v = (float *)p;
    p = take(4 * R * qd); if (w) w->attn = (float *)p;
    p = take(4 * R * c.ffn_dim); if (w) w->gate = (float *)p;
    p = take(4 * R * c.ffn_dim); if (w) w->up = (float *)p;
    p = take(4 * R * (size_t)c.vocab); if (w) w->logits = (float *)p;
    const size_t pf = m->path >= PV_PATH_MATRIX ? pv_mat_part_floats(m, rows_cap, units_cap, n_pages * m->cfg.page_tokens) : 0;
    p = take(4 * pf + 256); if (w) { w->part = (float *)p; w->part_floats = pf; }
    return off;
}

// Rows per prefill chunk: the widest block the kernels of this model have (the matrix path:
// PV_MAX_ROWS whatever max_gamma is; a prompt then needs a quarter of the passes over the
// weights that 16-row chunks would).  The workspace is sized for it.
static inline int prefill_rows_of(const pv_model *m)
{
    return (m->path >= PV_PATH_MATRIX && m->cfg.max_gamma < PV_MAX_ROWS) ? PV_MAX_ROWS : m->cfg.max_gamma;
}
static inline int rows_cap_of(const pv_model *m) { return (prefill_rows_of(m) + PV_ROW_PAD - 1) / PV_ROW_PAD * PV_ROW_PAD; }
// a workspace's attention partials: one sequence of rows_cap rows, or a batch (every further sequence rounds its rows up to whole units)
static inline int units_cap_of(const pv_model *m) { return m->path >= PV_PATH_MATRIX ? pv_attn_units(m, rows_cap_of(m)) + PV_MAX_SEQ - 1 : 0; }

extern "C" int pv_cache_bytes(const pv_model *m, int32_t max_tokens, size_t *page_pool_bytes, size_t *workspace_bytes)
{
    if (!m || !page_pool_bytes || !workspace_bytes) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (max_tokens <= 0) { pv_set_error("max_tokens must be positive"); return PV_ERANGE; }
    if ((max_tokens + m->cfg.page_tokens - 1) / m->cfg.page_tokens >= (1 << 26)) { pv_set_error("max_tokens %d: more than 2^26 pages", max_tokens); return PV_ERANGE; }
    const pv_model_config &c = m->cfg;
    const int n_pages = (max_tokens + c.page_tokens - 1) / c.page_tokens;
    *page_pool_bytes = align_up((size_t)c.n_layers * n_pages * c.n_kv_heads * 2 * c.page_tokens * c.head_dim * m->elt, 256);
    *workspace_bytes = layout_ws(m, rows_cap_of(m), units_cap_of(m), n_pages, nullptr, nullptr);
    return PV_OK;
}

extern "C" int pv_cache_create(const pv_model *m, void *d_page_pool, size_t page_pool_bytes, void *d_workspace,
                               size_t workspace_bytes, int32_t max_tokens, pv_cache **out)
{
    if (!m || !d_page_pool || !d_workspace || !out) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (((uintptr_t)d_page_pool | (uintptr_t)d_workspace) & 255) { pv_set_error("device buffers must be 256-byte aligned"); return PV_EINVAL; }
    size_t need_p, need_w;
    int rc = pv_cache_bytes(m, max_tokens, &need_p, &need_w);
    if (rc != PV_OK) return rc;
    if (page_pool_bytes < need_p || workspace_bytes < need_w) { pv_set_error("pool %zu < %zu or workspace %zu < %zu", page_pool_bytes, need_p, workspace_bytes, need_w); return PV_ENOMEM; }
    if (m->path >= PV_PATH_MATRIX && (rc = pv_mat_attention_init(m->cfg.head_dim)) != PV_OK) return rc;
    if (m->path >= PV_PATH_MATRIX && m->wbits == 4 && (rc = pv_mat_gemm_init()) != PV_OK) return rc;
    pv_cache *c = new (std::nothrow) pv_cache();
    if (!c) return PV_ENOMEM;
    c->m = m; c->d_pool = (char *)d_page_pool; c->pool_bytes = page_pool_bytes;
    c->d_ws = (char *)d_workspace; c->ws_bytes = workspace_bytes;
    c->max_tokens = max_tokens; c->n_pages = (max_tokens + m->cfg.page_tokens - 1) / m->cfg.page_tokens;
    c->rows_cap = rows_cap_of(m); c->units_cap = units_cap_of(m);
    layout_ws(m, c->rows_cap, c->units_cap, c->n_pages, &c->ws, c->d_ws);
    c->len = 0; c->pending = -1; c->last_rows = 0; c->blk_start = 0; c->blk_rows = 0; c->blk_units = 0; c->blk_seq_rows = 0; c->attn_keys = 0; c->in_flight = false; c->flight_stream = nullptr; c->io = nullptr;
    c->prof_kind = PV_PROF_NONE; c->prof_pending = 0; c->prof_ev = nullptr; c->prof_ms = 0; c->prof_launches = 0;
    c->use_graphs = true; c->cap_stream = nullptr;
    for (auto &row : c->gexec) for (auto &md : row) for (auto &ge : md) ge = nullptr;
    if (hipHostMalloc((void **)&c->io, sizeof(pv_host_io), hipHostMallocMapped | hipHostMallocCoherent) != hipSuccess) {
        pv_set_error("hipHostMalloc failed"); delete c; return PV_EHIP;
    }
    memset(c->io, 0, sizeof(pv_host_io));
    if (hipHostGetDevicePointer((void **)&c->d_io, c->io, 0) != hipSuccess) {
        pv_set_error("hipHostGetDevicePointer failed"); (void)hipHostFree(c->io); delete c; return PV_EHIP;
    }
    // device state, identity page table; activations zeroed once so padding rows are finite
    // pages start out as zeros so that never-written slots of a page can never hold NaN bit patterns
    hipError_t e = hipMemset(c->d_ws, 0, need_w);
    if (e == hipSuccess) e = hipMemset(c->d_pool, 0, need_p);
    int32_t *ident = (int32_t *)malloc(sizeof(int32_t) * c->n_pages);
    for (int i = 0; i < c->n_pages; ++i) ident[i] = i;
    if (e == hipSuccess) e = hipMemcpy(c->ws.page_table, ident, sizeof(int32_t) * c->n_pages, hipMemcpyHostToDevice);
    free(ident);
    pv_dev_state st; memset(&st, 0, sizeof(st)); st.pending = -1;
    // a plain step's block is one sequence: this cache
    c->io->single.n_seq = 1;
    c->io->single.seq[0].st = c->ws.state; c->io->single.seq[0].pool = c->d_pool; c->io->single.seq[0].page_table = c->ws.page_table;
    c->io->single.seq[0].gamma = 0; c->io->single.seq[0].row0 = 0; c->io->single.seq[0].n_pages = c->n_pages; c->io->single.seq[0].unit0 = 0;
    st.blk = c->io->single;
    if (e == hipSuccess) e = hipMemcpy(c->ws.state, &st, sizeof(st), hipMemcpyHostToDevice);
    if (e != hipSuccess) { pv_set_error("cache initialisation failed: %s", hipGetErrorString(e)); (void)hipHostFree(c->io); delete c; return PV_EHIP; }
    *out = c;
    return PV_OK;
}

extern "C" void pv_cache_destroy(pv_cache *c)
{
    if (!c) return;
    if (c->io) (void)hipHostFree(c->io);
    for (auto &row : c->gexec) for (auto &md : row) for (auto &ge : md) if (ge) (void)hipGraphExecDestroy(ge);
    if (c->cap_stream) (void)hipStreamDestroy(c->cap_stream);
    if (c->prof_ev) {
        for (int i = 0; i < 2 * c->m->cfg.n_layers; ++i) (void)hipEventDestroy(c->prof_ev[i]);
        free(c->prof_ev);
    }
    delete c;
}

extern "C" int pv_cache_set_page_table(pv_cache *c, const int32_t *phys_pages, int32_t n_pages, void *hip_stream)
{
    if (!c || !phys_pages) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (c->len != 0 || c->in_flight) { pv_set_error("page table can only be replaced on an empty, idle cache"); return PV_ESTATE; }
    if (n_pages != c->n_pages) { pv_set_error("n_pages %d != %d", n_pages, c->n_pages); return PV_EINVAL; }
    char *seen = (char *)calloc(n_pages, 1);
    for (int i = 0; i < n_pages; ++i) {
        if (phys_pages[i] < 0 || phys_pages[i] >= n_pages || seen[phys_pages[i]]) { free(seen); pv_set_error("page table is not a permutation"); return PV_EINVAL; }
        seen[phys_pages[i]] = 1;
    }
    free(seen);
    hipStream_t s = (hipStream_t)hip_stream;
    PV_HIP(hipMemcpyAsync(c->ws.page_table, phys_pages, sizeof(int32_t) * n_pages, hipMemcpyHostToDevice, s));
    PV_HIP(hipStreamSynchronize(s));
    return PV_OK;
}

// ---- the step ----

// the step's launches on stream s.  No copy nodes: the first kernel reads the draft ids from the
// pinned mailbox, the last one writes accepted_len, next_token and the error flag into it; the
// row count and the mode are kernel arguments (a recorded graph is keyed by them).
static int record_block(pv_cache *c, int rows, int mode, hipStream_t s)
{
    (void)rows; (void)mode;      // read by the kernel families from c->last_rows and c->io->hdr
    return c->m->path >= PV_PATH_MATRIX ? pv_mat_run_block(c, s) : pv_vec_run_block(c, s);
}

static int enqueue_block(pv_cache *c, const int32_t *tokens, int rows, int mode, hipStream_t s)
{
    const pv_model *m = c->m;
    for (int j = 0; j < rows; ++j)
        if (tokens[j] < 0 || tokens[j] >= m->cfg.vocab) { pv_set_error("token id %d at position %d outside [0, %d)", tokens[j], j, m->cfg.vocab); return PV_ERANGE; }
    memcpy(c->io->draft, tokens, sizeof(int32_t) * rows);
    c->io->hdr[2] = rows; c->io->hdr[3] = mode;
    c->last_rows = rows;
    c->blk_start = c->len; c->blk_rows = rows;
    // The launch sequence depends on (rows, mode) only: everything else a kernel needs (length,
    // pending token, draft ids) it reads from device memory.  So the sequence is recorded once
    // per (rows, mode) as a HIP graph and replayed; instrumented steps run the plain launches.
    c->attn_keys = c->len + rows;
    if (c->use_graphs && c->prof_kind == PV_PROF_NONE) {
        // a recorded step serves every length up to the next power of two: its attention grid is sized for that
        int bucket = 8;
        while ((1 << bucket) < c->len + rows && bucket < 30) ++bucket;
        c->attn_keys = 1 << bucket;
        hipGraphExec_t &ge = c->gexec[rows][mode][bucket - 8];
        if (!ge) {
            if (!c->cap_stream) PV_HIP(hipStreamCreateWithFlags(&c->cap_stream, hipStreamNonBlocking));
            PV_HIP(hipStreamBeginCapture(c->cap_stream, hipStreamCaptureModeThreadLocal));
            const int rrc = record_block(c, rows, mode, c->cap_stream);
            hipGraph_t g = nullptr;
            const hipError_t e = hipStreamEndCapture(c->cap_stream, &g);
            if (rrc != PV_OK) { if (g) (void)hipGraphDestroy(g); return rrc; }
            if (e != hipSuccess || !g) { pv_set_error("stream capture of the step failed: %s", hipGetErrorString(e)); return PV_EHIP; }
            const hipError_t ei = hipGraphInstantiate(&ge, g, nullptr, nullptr, 0);
            (void)hipGraphDestroy(g);
            if (ei != hipSuccess) { ge = nullptr; pv_set_error("hipGraphInstantiate failed: %s", hipGetErrorString(ei)); return PV_EHIP; }
        }
        PV_HIP(hipGraphLaunch(ge, s));
        return PV_OK;
    }
    return record_block(c, rows, mode, s);
}

int pv_prof_mark(pv_cache *c, int kind, int slot, int end, hipStream_t s)
{
    if (c->prof_kind != kind) return PV_OK;
    PV_HIP(hipEventRecord(c->prof_ev[2 * slot + end], s));
    if (end && slot + 1 > c->prof_pending) c->prof_pending = slot + 1;
    return PV_OK;
}

// after the step's stream has been synchronised: fold the event pairs into the counters
static void prof_collect(pv_cache *c)
{
    for (int i = 0; i < c->prof_pending; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, c->prof_ev[2 * i], c->prof_ev[2 * i + 1]) == hipSuccess) { c->prof_ms += ms; c->prof_launches += 1; }
    }
    c->prof_pending = 0;
}

extern "C" int pv_cache_use_graphs(pv_cache *c, int32_t enable)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    c->use_graphs = enable != 0;
    return PV_OK;
}

extern "C" int pv_profile_select(pv_cache *c, int32_t which)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    if (which < PV_PROF_NONE || which > PV_PROF_LMHEAD) { pv_set_error("bad kernel selector %d", which); return PV_EINVAL; }
    if (which != PV_PROF_NONE && !c->prof_ev) {
        const int n = 2 * c->m->cfg.n_layers;
        c->prof_ev = (hipEvent_t *)calloc(n, sizeof(hipEvent_t));
        if (!c->prof_ev) return PV_ENOMEM;
        for (int i = 0; i < n; ++i) PV_HIP(hipEventCreate(&c->prof_ev[i]));
    }
    c->prof_kind = which; c->prof_pending = 0; c->prof_ms = 0; c->prof_launches = 0;
    return PV_OK;
}

extern "C" int pv_profile_read(pv_cache *c, double *total_ms, int64_t *launches, uint64_t *bytes_per_launch)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    const pv_model_config &f = c->m->cfg;
    const uint64_t e = c->m->elt, d = f.d_model, qd = (uint64_t)f.n_q_heads * f.head_dim, kvd = (uint64_t)f.n_kv_heads * f.head_dim;
    uint64_t b = 0;
    switch (c->prof_kind) {
    case PV_PROF_QKV: b = (qd + 2 * kvd) * d * e; break;
    case PV_PROF_ATTENTION: b = 2 * kvd * e * (uint64_t)c->len; break;
    case PV_PROF_OPROJ: b = d * qd * e; break;
    case PV_PROF_GATEUP: b = 2 * (uint64_t)f.ffn_dim * d * e; break;
    case PV_PROF_DOWN: b = (uint64_t)f.ffn_dim * d * e; break;
    case PV_PROF_LMHEAD: b = (uint64_t)f.vocab * d * e; break;
    default: break;
    }
    if (c->m->wbits == 4 && c->prof_kind != PV_PROF_ATTENTION) b = b / (16 * 128 * e) * PV_Q4_BATCH;   // 16 x 128 weights per batch
    if (total_ms) *total_ms = c->prof_ms;
    if (launches) *launches = c->prof_launches;
    if (bytes_per_launch) *bytes_per_launch = b;
    return PV_OK;
}

__global__ void __launch_bounds__(256) k_calib_copy(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

extern "C" int pv_calib_copy(void *d_dst, const void *d_src, size_t nbytes, void *hip_stream)
{
    if (!d_dst || !d_src || (nbytes & 15) || (((uintptr_t)d_dst | (uintptr_t)d_src) & 15)) {
        pv_set_error("pv_calib_copy: pointers and size must be multiples of 16 bytes"); return PV_EINVAL;
    }
    const size_t n = nbytes / 16;
    if (n == 0) return PV_OK;
    const unsigned grid = (unsigned)((n + 255) / 256 < 8192 ? (n + 255) / 256 : 8192);
    k_calib_copy<<<grid, 256, 0, (hipStream_t)hip_stream>>>((uint4 *)d_dst, (const uint4 *)d_src, n);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

// after the step's stream has been synchronised: fold the step's results into the host mirror
// every wave streams a contiguous slice of `tiles` 1 KiB tiles (64 lanes x 16 bytes), eight loads in
// flight per lane; the rest of the region is read by the first waves, one tile each
typedef __attribute__((ext_vector_type(4))) unsigned int calib_u32x4;
__device__ inline uint4 calib_load(const uint4 *p)
{
#ifdef PV_CALIB_PLAIN
    return *p;
#else
    const calib_u32x4 v = __builtin_nontemporal_load((const calib_u32x4 *)p);   // read once, like the weight streams it is compared with
    return make_uint4(v.x, v.y, v.z, v.w);
#endif
}

__global__ void __launch_bounds__(512) k_calib_read(const uint4 *__restrict__ src, size_t tiles, size_t n, uint4 *sink)
{
    const int lane = threadIdx.x & 63;
    const size_t wave = (size_t)blockIdx.x * 8 + (threadIdx.x >> 6), nwaves = (size_t)gridDim.x * 8;
    const uint4 *q = src + wave * tiles * 64 + lane;
    uint4 acc = make_uint4(0u, 0u, 0u, 0u);
    for (size_t t = 0; t < tiles; t += 8) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = calib_load(&q[(t + u) * 64]);
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    for (size_t i = nwaves * tiles * 64 + wave * 64 + lane; i < n; i += nwaves * 64) { const uint4 v = src[i]; acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w; }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u && acc.w == 0x87654321u) sink[0] = acc;
}

extern "C" int pv_calib_read(const void *d_src, size_t nbytes, void *d_sink, void *hip_stream)
{
    if (!d_src || !d_sink || (nbytes & 15) || (((uintptr_t)d_src | (uintptr_t)d_sink) & 15)) {
        pv_set_error("pv_calib_read: pointers and size must be multiples of 16 bytes"); return PV_EINVAL;
    }
    const size_t n = nbytes / 16;
    if (n == 0) return PV_OK;
    const unsigned grid = 1024;
    const size_t tiles = n / ((size_t)grid * 8 * 64) / 8 * 8;
    k_calib_read<<<grid, 512, 0, (hipStream_t)hip_stream>>>((const uint4 *)d_src, tiles, n, (uint4 *)d_sink);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

static int absorb_result(pv_cache *c)
{
    prof_collect(c);
    c->len += c->io->result[0];
    c->pending = c->io->result[1];
    if (c->io->result[PV_RESULT_ERR]) { pv_set_error("a row of the block has no finite logit (non-finite weights or activations); nothing was committed"); return PV_ENUMERIC; }
    return PV_OK;
}

static int check_ready(const pv_cache *c)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache; call pv_verify_wait first"); return PV_ESTATE; }
    if (!model_complete(c->m)) { pv_set_error("not all weights have been loaded"); return PV_ESTATE; }
    return PV_OK;
}

extern "C" int pv_prefill(pv_cache *c, const int32_t *tokens, int32_t n, void *hip_stream)
{
    int rc = check_ready(c);
    if (rc != PV_OK) return rc;
    if (!tokens) { pv_set_error("null tokens"); return PV_EINVAL; }
    if (n <= 0 || c->len + n > c->max_tokens) { pv_set_error("prefill of %d tokens does not fit (length %d, max %d)", n, c->len, c->max_tokens); return PV_ERANGE; }
    for (int j = 0; j < n; ++j)
        if (tokens[j] < 0 || tokens[j] >= c->m->cfg.vocab) { pv_set_error("token id %d at position %d outside [0, %d)", tokens[j], j, c->m->cfg.vocab); return PV_ERANGE; }
    hipStream_t s = (hipStream_t)hip_stream;
    const int chunk = prefill_rows_of(c->m);
    for (int off = 0; off < n; off += chunk) {
        const int rows = n - off < chunk ? n - off : chunk;
        const bool last = off + rows >= n;
        rc = enqueue_block(c, tokens + off, rows, last ? PV_MODE_PREFILL_LAST : PV_MODE_PREFILL_MID, s);
        if (rc != PV_OK) return rc;
        PV_HIP(hipStreamSynchronize(s));          // the mailbox is reused by the next chunk
        if ((rc = absorb_result(c)) != PV_OK) return rc;
    }
    return PV_OK;
}

static int verify_checks(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma)
{
    int rc = check_ready(c);
    if (rc != PV_OK) return rc;
    if (!draft) { pv_set_error("null draft"); return PV_EINVAL; }
    if (prefix_len != c->len) { pv_set_error("prefix_len %d != cache length %d", prefix_len, c->len); return PV_ESTATE; }
    if (gamma < 1 || gamma > c->m->cfg.max_gamma) { pv_set_error("gamma %d outside [1, %d]", gamma, c->m->cfg.max_gamma); return PV_ERANGE; }
    if (c->len + gamma > c->max_tokens) { pv_set_error("length %d + gamma %d exceeds max_tokens %d", c->len, gamma, c->max_tokens); return PV_ERANGE; }
    return PV_OK;
}

extern "C" int pv_verify_async(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma, void *hip_stream)
{
    int rc = verify_checks(c, prefix_len, draft, gamma);
    if (rc != PV_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    rc = enqueue_block(c, draft, gamma, PV_MODE_VERIFY, s);
    if (rc != PV_OK) return rc;
    c->in_flight = true; c->flight_stream = s;
    return PV_OK;
}

// ---- the step for callers that may not allocate ----
//
// One fixed device array stands in for the per-step part of the cache's workspace (activations,
// operands, partial sums, logits, arg-max candidates).  In host code the array's name is only a
// stand-in for the symbol: its device address is looked up once per device and kept.
#define PV_MAX_DEVICES 64
static __device__ __align__(256) unsigned char scratch[PV_STATIC_SCRATCH_BYTES];
static char *g_scratch_ptr[PV_MAX_DEVICES];
static std::mutex g_scratch_mu;

static int static_scratch(char **out)
{
    int dev = -1;
    PV_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= PV_MAX_DEVICES) { pv_set_error("device index %d outside [0, %d)", dev, PV_MAX_DEVICES); return PV_EINVAL; }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        PV_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));      // this device's copy of the array
        if (!p) { pv_set_error("hipGetSymbolAddress returned a null address"); return PV_EHIP; }
        g_scratch_ptr[dev] = (char *)p;
    }
    *out = g_scratch_ptr[dev];
    return PV_OK;
}

__global__ void __launch_bounds__(256) k_zero(uint4 *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = make_uint4(0u, 0u, 0u, 0u);
}

extern "C" int pv_verify_async_static(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma, void *hip_stream)
{
    int rc = verify_checks(c, prefix_len, draft, gamma);
    if (rc != PV_OK) return rc;
    if (c->prof_kind != PV_PROF_NONE) { pv_set_error("kernel instrumentation is switched on for this cache"); return PV_ESTATE; }
    const pv_model *m = c->m;
    // per-step buffers for a block of this size, laid out in the fixed array (the same layout routine
    // as a workspace; the cache state and the page table stay where the cache keeps them)
    const int cap = (gamma + PV_ROW_PAD - 1) / PV_ROW_PAD * PV_ROW_PAD;
    const int ucap = m->path >= PV_PATH_MATRIX ? pv_attn_units(m, cap) : 0;          // one sequence: no batch allowance
    const size_t need = layout_ws(m, cap, ucap, c->n_pages, nullptr, nullptr);
    if (need > PV_STATIC_SCRATCH_BYTES) {
        pv_set_error("a %d-row step of this model with max_tokens %d needs %zu bytes of per-step buffers, the fixed array holds %zu",
                     gamma, c->max_tokens, need, (size_t)PV_STATIC_SCRATCH_BYTES);
        return PV_ENOMEM;
    }
    char *base = nullptr;
    if ((rc = static_scratch(&base)) != PV_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    // the array keeps the last call's contents (of any cache, any model): start from zeros, as a fresh workspace does
    k_zero<<<1024, 256, 0, s>>>((uint4 *)base, need / 16);
    PV_HIP(hipGetLastError());
    const pv_ws own = c->ws;
    const int own_cap = c->rows_cap, own_ucap = c->units_cap;
    layout_ws(m, cap, ucap, c->n_pages, &c->ws, base);
    c->ws.state = own.state; c->ws.page_table = own.page_table;
    c->rows_cap = cap; c->units_cap = ucap;
    for (int j = 0; j < gamma; ++j)
        if (draft[j] < 0 || draft[j] >= m->cfg.vocab) { c->ws = own; c->rows_cap = own_cap; c->units_cap = own_ucap; pv_set_error("token id %d at position %d outside [0, %d)", draft[j], j, m->cfg.vocab); return PV_ERANGE; }
    memcpy(c->io->draft, draft, sizeof(int32_t) * gamma);
    c->io->hdr[2] = gamma; c->io->hdr[3] = PV_MODE_VERIFY;
    c->last_rows = gamma;
    c->blk_start = c->len; c->blk_rows = gamma;
    c->attn_keys = c->len + gamma;
    rc = record_block(c, gamma, PV_MODE_VERIFY, s);      // plain launches: the kernels take the buffers as arguments
    c->ws = own; c->rows_cap = own_cap; c->units_cap = own_ucap;
    c->last_rows = 0;                                   // the block's logits are in the shared array: not kept for pv_debug_logits
    if (rc != PV_OK) return rc;
    c->in_flight = true; c->flight_stream = s;
    return PV_OK;
}

extern "C" int pv_verify_wait(pv_cache *c, int32_t *accepted_len, int32_t *next_token)
{
    if (!c || !accepted_len || !next_token) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (!c->in_flight) { pv_set_error("no verify in flight"); return PV_ESTATE; }
    c->in_flight = false;
    PV_HIP(hipStreamSynchronize(c->flight_stream));
    const int rc = absorb_result(c);
    *accepted_len = c->io->result[0];
    *next_token = c->io->result[1];
    return rc;
}

extern "C" int pv_verify(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma,
                         int32_t *accepted_len, int32_t *next_token, void *hip_stream)
{
    if (!accepted_len || !next_token) { pv_set_error("null output pointer"); return PV_EINVAL; }
    int rc = pv_verify_async(c, prefix_len, draft, gamma, hip_stream);
    if (rc != PV_OK) return rc;
    return pv_verify_wait(c, accepted_len, next_token);
}

// ---- several sequences in one pass over the weights ----
extern "C" int pv_verify_batch(pv_cache *const *caches, int32_t n_seq, const int32_t *prefix_len, const int32_t *draft,
                               const int32_t *gamma, int32_t *accepted_len, int32_t *next_token, void *hip_stream)
{
    if (!caches || !prefix_len || !draft || !gamma || !accepted_len || !next_token) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (n_seq < 1 || n_seq > PV_MAX_SEQ) { pv_set_error("n_seq %d outside [1, %d]", n_seq, PV_MAX_SEQ); return PV_ERANGE; }
    pv_cache *lead = caches[0];
    int rc = check_ready(lead);
    if (rc != PV_OK) return rc;
    const pv_model *m = lead->m;
    if (m->path < PV_PATH_MATRIX) { pv_set_error("batched verification runs on the matrix path (bf16 models)"); return PV_EINVAL; }
    if (lead->prof_kind != PV_PROF_NONE) { pv_set_error("kernel instrumentation is switched on for the first cache"); return PV_ESTATE; }
    int rows = 0, units = 0, seq_rows = 0;
    for (int i = 0; i < n_seq; ++i) {
        pv_cache *c = caches[i];
        if (!c) { pv_set_error("null cache %d", i); return PV_EINVAL; }
        for (int k = 0; k < i; ++k) if (caches[k] == c) { pv_set_error("cache %d appears twice in the batch", i); return PV_EINVAL; }
        if (c->m != m) { pv_set_error("cache %d belongs to another model", i); return PV_EINVAL; }
        if (c->max_tokens != lead->max_tokens) { pv_set_error("caches of a batch must have the same max_tokens (%d vs %d)", c->max_tokens, lead->max_tokens); return PV_EINVAL; }
        if ((rc = verify_checks(c, prefix_len[i], draft + rows, gamma[i])) != PV_OK) return rc;
        rows += gamma[i];
    }
    if (rows > lead->rows_cap) { pv_set_error("%d rows in all: a step of this model takes at most %d", rows, lead->rows_cap); return PV_ERANGE; }
    for (int j = 0; j < rows; ++j)
        if (draft[j] < 0 || draft[j] >= m->cfg.vocab) { pv_set_error("token id %d at row %d outside [0, %d)", draft[j], j, m->cfg.vocab); return PV_ERANGE; }
    // the block's description: rows and attention row-group units of every sequence, in order
    pv_block_desc &bd = lead->io->batch;
    bd.n_seq = n_seq;
    int r0 = 0;
    for (int i = 0; i < n_seq; ++i) {
        pv_cache *c = caches[i];
        pv_seq_ref &sq = bd.seq[i];
        sq.st = c->ws.state; sq.pool = c->d_pool; sq.page_table = c->ws.page_table;
        sq.gamma = gamma[i]; sq.row0 = r0; sq.n_pages = c->n_pages; sq.unit0 = units;
        r0 += gamma[i];
        units += pv_attn_units(m, gamma[i]);
        if (gamma[i] > seq_rows) seq_rows = gamma[i];
    }
    if (units > lead->units_cap) { pv_set_error("the batch needs %d attention row groups, the workspace holds %d", units, lead->units_cap); return PV_ENOMEM; }
    memcpy(lead->io->draft, draft, sizeof(int32_t) * rows);
    lead->io->hdr[2] = rows; lead->io->hdr[3] = PV_MODE_VERIFY;
    hipStream_t s = (hipStream_t)hip_stream;
    // description in, the step as plain launches, the cache's own one-sequence description back in
    PV_HIP(hipMemcpyAsync(&lead->ws.state->blk, &bd, sizeof(pv_block_desc), hipMemcpyHostToDevice, s));
    lead->last_rows = rows; lead->blk_units = units; lead->blk_seq_rows = seq_rows;
    lead->attn_keys = 0;
    for (int i = 0; i < n_seq; ++i) if (caches[i]->len + gamma[i] > lead->attn_keys) lead->attn_keys = caches[i]->len + gamma[i];
    rc = record_block(lead, rows, PV_MODE_VERIFY, s);
    lead->blk_units = 0; lead->blk_seq_rows = 0;
    const hipError_t e1 = hipMemcpyAsync(&lead->ws.state->blk, &lead->io->single, sizeof(pv_block_desc), hipMemcpyHostToDevice, s);
    const hipError_t e2 = hipStreamSynchronize(s);
    if (rc != PV_OK) return rc;
    if (e1 != hipSuccess || e2 != hipSuccess) { pv_set_error("batched step failed: %s", hipGetErrorString(e1 != hipSuccess ? e1 : e2)); return PV_EHIP; }
    for (int i = 0; i < n_seq; ++i) {
        pv_cache *c = caches[i];
        accepted_len[i] = lead->io->result[2 * i]; next_token[i] = lead->io->result[2 * i + 1];
        c->blk_start = c->len; c->blk_rows = gamma[i];
        c->len += accepted_len[i]; c->pending = next_token[i];
        if (c != lead) c->last_rows = 0;
    }
    if (lead->io->result[PV_RESULT_ERR]) { pv_set_error("a row of the block has no finite logit (non-finite weights or activations)"); return PV_ENUMERIC; }
    return PV_OK;
}

// ---- a draft tree instead of a draft chain ----
static_assert(offsetof(pv_host_io, parent) == sizeof(int32_t) * PV_MAX_ROWS, "the block set-up kernel finds the parents right behind the draft ids");

extern "C" int pv_verify_tree(pv_cache *c, int32_t prefix_len, const int32_t *tokens, const int32_t *parent, int32_t n,
                              int32_t *accepted_len, int32_t *next_token, int32_t *path, void *hip_stream)
{
    int rc = check_ready(c);
    if (rc != PV_OK) return rc;
    if (!tokens || !parent || !accepted_len || !next_token) { pv_set_error("null pointer"); return PV_EINVAL; }
    const pv_model *m = c->m;
    if (m->path < PV_PATH_MATRIX) { pv_set_error("draft trees run on the matrix path (bf16 models)"); return PV_EINVAL; }
    if (c->prof_kind != PV_PROF_NONE) { pv_set_error("kernel instrumentation is switched on for this cache"); return PV_ESTATE; }
    if (prefix_len != c->len) { pv_set_error("prefix_len %d != cache length %d", prefix_len, c->len); return PV_ESTATE; }
    if (n < 1 || n > c->rows_cap || n > PV_MAX_ROWS) { pv_set_error("a draft tree has 1 .. %d nodes, got %d", c->rows_cap < PV_MAX_ROWS ? c->rows_cap : PV_MAX_ROWS, n); return PV_ERANGE; }
    if (c->len + n > c->max_tokens) { pv_set_error("length %d + %d nodes exceeds max_tokens %d", c->len, n, c->max_tokens); return PV_ERANGE; }
    for (int i = 0; i < n; ++i) {
        if (tokens[i] < 0 || tokens[i] >= m->cfg.vocab) { pv_set_error("token id %d at node %d outside [0, %d)", tokens[i], i, m->cfg.vocab); return PV_ERANGE; }
        if (parent[i] < -1 || parent[i] >= i) { pv_set_error("node %d: parent %d must be -1 or an earlier node", i, parent[i]); return PV_EINVAL; }
    }
    memcpy(c->io->draft, tokens, sizeof(int32_t) * n);
    memcpy(c->io->parent, parent, sizeof(int32_t) * n);
    c->io->hdr[2] = n; c->io->hdr[3] = PV_MODE_TREE;
    c->last_rows = n; c->attn_keys = c->len + n;
    hipStream_t s = (hipStream_t)hip_stream;
    rc = record_block(c, n, PV_MODE_TREE, s);               // plain launches
    if (rc == PV_OK) rc = pv_k_tree_compact(c, s);
    const hipError_t e = hipStreamSynchronize(s);
    if (rc != PV_OK) return rc;
    if (e != hipSuccess) { pv_set_error("draft-tree step failed: %s", hipGetErrorString(e)); return PV_EHIP; }
    c->blk_rows = 0;                                         // the rows off the path are gone: nothing to re-admit
    rc = absorb_result(c);
    *accepted_len = c->io->result[0];
    *next_token = c->io->result[1];
    if (path && rc == PV_OK) {
        // the accepted rows, in order (device state -> host)
        PV_HIP(hipMemcpy(path, c->ws.state->path, sizeof(int32_t) * (size_t)*accepted_len, hipMemcpyDeviceToHost));
    }
    return rc;
}

extern "C" int pv_rollback(pv_cache *c, int32_t new_len, void *hip_stream)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    if (new_len < 0 || new_len > c->len) { pv_set_error("new_len %d outside [0, %d]", new_len, c->len); return PV_ERANGE; }
    hipStream_t s = (hipStream_t)hip_stream;
    int rc = pv_k_set_state(c, new_len, -1, s);
    if (rc != PV_OK) return rc;
    PV_HIP(hipStreamSynchronize(s));
    c->len = new_len; c->pending = -1; c->blk_rows = 0;
    return PV_OK;
}

extern "C" int pv_cache_readmit(pv_cache *c, int32_t new_len, int32_t pending, void *hip_stream)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    if (c->blk_rows == 0) { pv_set_error("no block on record to re-admit from"); return PV_ESTATE; }
    if (new_len < c->len || new_len > c->blk_start + c->blk_rows) { pv_set_error("new_len %d outside [%d, %d]", new_len, c->len, c->blk_start + c->blk_rows); return PV_ERANGE; }
    if (pending < -1 || pending >= c->m->cfg.vocab) { pv_set_error("token %d out of range", pending); return PV_ERANGE; }
    hipStream_t s = (hipStream_t)hip_stream;
    int rc = pv_k_set_state(c, new_len, pending, s);
    if (rc != PV_OK) return rc;
    PV_HIP(hipStreamSynchronize(s));
    c->len = new_len; c->pending = pending;
    return PV_OK;
}

extern "C" int pv_cache_len(const pv_cache *c, int32_t *len, int32_t *pending)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (len) *len = c->len;
    if (pending) *pending = c->pending;
    return PV_OK;
}

extern "C" int pv_cache_set_pending(pv_cache *c, int32_t token, void *hip_stream)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    if (token < -1 || token >= c->m->cfg.vocab) { pv_set_error("token %d out of range", token); return PV_ERANGE; }
    hipStream_t s = (hipStream_t)hip_stream;
    int rc = pv_k_set_state(c, c->len, token, s);
    if (rc != PV_OK) return rc;
    PV_HIP(hipStreamSynchronize(s));
    c->pending = token;
    return PV_OK;
}

extern "C" int pv_debug_logits(pv_cache *c, float *host_out, int32_t *rows, void *hip_stream)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    if (rows) *rows = c->last_rows;
    if (!host_out || c->last_rows == 0) return PV_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    PV_HIP(hipMemcpyAsync(host_out, c->ws.logits, sizeof(float) * (size_t)c->last_rows * c->m->cfg.vocab, hipMemcpyDeviceToHost, s));
    PV_HIP(hipStreamSynchronize(s));
    return PV_OK;
}

extern "C" int pv_debug_pred(pv_cache *c, int32_t *host_out, int32_t *rows, void *hip_stream)
{
    if (!c) { pv_set_error("null cache"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    if (rows) *rows = c->last_rows;
    if (!host_out || c->last_rows == 0) return PV_OK;
    hipStream_t s = (hipStream_t)hip_stream;
    PV_HIP(hipMemcpyAsync(host_out, c->ws.state->pred, sizeof(int32_t) * c->last_rows, hipMemcpyDeviceToHost, s));
    PV_HIP(hipStreamSynchronize(s));
    return PV_OK;
}

extern "C" int pv_cache_export(pv_cache *c, void *host_out, size_t nbytes, void *hip_stream)
{
    if (!c || !host_out) { pv_set_error("null pointer"); return PV_EINVAL; }
    if (c->in_flight) { pv_set_error("a verify is in flight on this cache"); return PV_ESTATE; }
    const pv_model_config &f = c->m->cfg;
    const size_t total = (size_t)f.n_layers * 2 * c->len * f.n_kv_heads * f.head_dim;
    if (nbytes < total * c->m->elt) { pv_set_error("export needs %zu bytes, got %zu", total * c->m->elt, nbytes); return PV_ENOMEM; }
    // bounce through the logits buffer (dead between steps) in chunks
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t cap = (size_t)c->rows_cap * f.vocab * sizeof(float) / c->m->elt;
    for (size_t e0 = 0; e0 < total; e0 += cap) {
        const size_t n = total - e0 < cap ? total - e0 : cap;
        int rc = pv_k_export(c, e0, n, c->ws.logits, s);
        if (rc != PV_OK) return rc;
        PV_HIP(hipMemcpyAsync((char *)host_out + e0 * c->m->elt, c->ws.logits, n * c->m->elt, hipMemcpyDeviceToHost, s));
        PV_HIP(hipStreamSynchronize(s));
    }
    c->last_rows = 0;           // the logits buffer no longer holds a block's logits
    c->blk_rows = 0;
    return PV_OK;
}

extern "C" int pv_step_bytes(const pv_cache *c, int32_t gamma, uint64_t *bytes)
{
    if (!c || !bytes) { pv_set_error("null pointer"); return PV_EINVAL; }
    const pv_model *m = c->m;
    const pv_model_config &f = m->cfg;
    uint64_t w = 0;
    for (int k = 0; k < PV_T_NKINDS; ++k) {
        if (k == PV_T_EMBED) continue;
        int64_t r, cc; tensor_dims(&f, k, &r, &cc);
        const bool global = k == PV_T_FINAL_NORM || k == PV_T_LM_HEAD;
        const uint64_t tb = (m->wbits == 4 && pv_is_q4_kind(k)) ? (uint64_t)(r / 16) * (cc / 128) * PV_Q4_BATCH : (uint64_t)r * cc * m->elt;
        w += tb * (global ? 1 : f.n_layers);
    }
    const uint64_t kv_tok = (uint64_t)f.n_layers * 2 * f.n_kv_heads * f.head_dim * m->elt;
    *bytes = w + kv_tok * (uint64_t)(c->len + gamma) + kv_tok * (uint64_t)gamma;
    return PV_OK;
}
