// Kernel wrappers of the attention units (pv_attention_body.h) for the per-kernel step sequence.
#include "pv_attention_body.h"

template <int HD, int TILES>
__global__ void __launch_bounds__(512)
k_attn(const attn_args a)
{
    extern __shared__ float4 smem4[];               // attn_smem_floats<HD>() floats: above the static limit for HD = 128
    attn_chunk<HD, TILES>(a, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z, (float *)smem4);
}

template <int NB, int HD>
__global__ void __launch_bounds__(256)
k_attn_merge(const attn_args a, int n_units)
{
    __shared__ float smem[256 + (256 / (HD / 4)) * (HD / 4) * 5];
    if ((int)blockIdx.x >= a.st->gamma) return;
    attn_merge_unit<NB, HD, 256>(a, blockIdx.x, blockIdx.y, n_units, threadIdx.x, smem);
}

// ------------------------------- host side ----------------------------------------

// Row-group units (32 query rows of one kv head) of one sequence with `rows` block rows
int pv_attn_units(const pv_model *m, int rows)
{
    const int group = m->cfg.n_q_heads / m->cfg.n_kv_heads;
    return (group * rows + 31) / 32;
}

size_t pv_attn_part_floats(const pv_model *m, int units_cap, int max_tokens)
{
    const pv_model_config &f = m->cfg;
    const int chunks = (max_tokens + 127) / 128;   // the finer of the two chunkings
    return (size_t)f.n_kv_heads * units_cap * chunks * 32 * (f.head_dim + 2);
}

// rows: rows of the block; a batched step also gives its unit count and the most rows any one sequence has
template <int NB, int HD>
static int launch(pv_cache *c, attn_args &a, int rows, hipStream_t s)
{
    const pv_model_config &f = c->m->cfg;
    const int seq_rows = c->blk_units ? c->blk_seq_rows : rows;
    const int nrows = a.group * seq_rows, units = c->blk_units ? c->blk_units : (nrows + 31) / 32;
    // up to 16 query rows per kv head: 256-key chunks, eight waves of 32 keys each; more rows:
    // 128-key chunks, the waves split into two 16-row tiles x four 32-key groups
    constexpr size_t lds = attn_smem_floats<HD>() * sizeof(float);
    // chunks to launch: enough for the keys this step can reach (the host's bound), not for the whole cache
    const int keys = c->attn_keys > 0 && c->attn_keys < c->max_tokens ? c->attn_keys : c->max_tokens;
    if (nrows <= 16) {
        a.chunk_shift = 8; a.max_chunks = (c->max_tokens + 255) / 256;
        k_attn<HD, 1><<<dim3((keys + 255) / 256, f.n_kv_heads, units), 512, lds, s>>>(a);
    } else {
        a.chunk_shift = 7; a.max_chunks = (c->max_tokens + 127) / 128;
        k_attn<HD, 2><<<dim3((keys + 127) / 128, f.n_kv_heads, units), 512, lds, s>>>(a);
    }
    PV_HIP(hipGetLastError());
    k_attn_merge<NB, HD><<<dim3(rows, f.n_q_heads), 256, 0, s>>>(a, units);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

template <int HD>
static int allow_lds()
{
    constexpr int lds = attn_smem_floats<HD>() * (int)sizeof(float);
    PV_HIP(hipFuncSetAttribute((const void *)k_attn<HD, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    PV_HIP(hipFuncSetAttribute((const void *)k_attn<HD, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, lds));
    return PV_OK;
}

// once per device before the first launch (and outside any stream capture): the attention
// kernels use more dynamic LDS than the default limit
int pv_mat_attention_init(int head_dim)
{
    switch (head_dim) {
    case 32: return allow_lds<32>();
    case 64: return allow_lds<64>();
    case 128: return allow_lds<128>();
    default: pv_set_error("matrix path: unsupported head_dim %d", head_dim); return PV_EINVAL;
    }
}

// q (bf16 hi + lo, rotated) -> xop_o; part = scratch of pv_attn_part_floats floats
int pv_mat_attention(pv_cache *c, int layer, int rows, float *part, uint16_t *xop_o, hipStream_t s)
{
    const pv_model_config &f = c->m->cfg;
    attn_args a;
    a.st = c->ws.state; a.page_table = c->ws.page_table; a.q_hi = (const uint16_t *)c->ws.q; a.q_lo = a.q_hi + (size_t)c->rows_cap * f.n_q_heads * f.head_dim; a.pool = (const uint16_t *)c->d_pool;
    a.geom = pv_geom(c); a.layer = layer; a.n_q_heads = f.n_q_heads; a.group = f.n_q_heads / f.n_kv_heads;
    a.max_chunks = (c->max_tokens + 127) / 128;        // sizes the partial arrays; the launch sets the chunking in use
    a.chunk_shift = 7;
    a.scale = 1.0f / sqrtf((float)f.head_dim);
    a.part_o = part;
    a.part_ml = part + (size_t)f.n_kv_heads * c->units_cap * a.max_chunks * 32 * f.head_dim;
    a.xop_o = xop_o; a.n_pages = c->n_pages; a.lo_off = pv_lo_off(rows);
    const bool nb1 = rows <= 8;
    switch (f.head_dim) {
    case 32: return nb1 ? launch<1, 32>(c, a, rows, s) : launch<2, 32>(c, a, rows, s);
    case 64: return nb1 ? launch<1, 64>(c, a, rows, s) : launch<2, 64>(c, a, rows, s);
    case 128: return nb1 ? launch<1, 128>(c, a, rows, s) : launch<2, 128>(c, a, rows, s);
    default: pv_set_error("matrix path: unsupported head_dim %d", f.head_dim); return PV_EINVAL;
    }
}
