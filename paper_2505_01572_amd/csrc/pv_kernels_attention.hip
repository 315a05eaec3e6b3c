// Kernel wrappers of the attention units (pv_attention_body.h) for the per-kernel step sequence.
#include "pv_attention_body.h"

template <int HD, int R>
__global__ void __launch_bounds__(512)
k_attn(const attn_args a)
{
    __shared__ float smem[attn_smem_floats<HD, R, 2>()];
    attn_chunk<HD, R, 2>(a, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.z, smem);
}

template <int NB, int HD>
__global__ void __launch_bounds__(256)
k_attn_merge(const attn_args a, int mp_count)
{
    __shared__ float smem[256 + (256 / (HD / 4)) * (HD / 4) * 5];
    if ((int)blockIdx.x >= a.st->gamma) return;
    attn_merge_unit<NB, HD, 256>(a, blockIdx.x, blockIdx.y, mp_count, threadIdx.x, smem);
}

// ------------------------------- host side ----------------------------------------

size_t pv_attn_part_floats(const pv_model *m, int rows_cap, int max_tokens)
{
    const pv_model_config &f = m->cfg;
    const int group = f.n_q_heads / f.n_kv_heads, mp = (group * rows_cap + 31) / 32, chunks = (max_tokens + 255) / 256;
    return (size_t)f.n_kv_heads * mp * chunks * 32 * (f.head_dim + 2);
}

template <int NB, int HD>
static int launch(pv_cache *c, attn_args &a, int rows, hipStream_t s)
{
    const pv_model_config &f = c->m->cfg;
    const int nrows = a.group * rows, mp = (nrows + 31) / 32;
    const dim3 grid(a.max_chunks, f.n_kv_heads, mp);
    if (nrows <= 16) k_attn<HD, 1><<<grid, 512, 0, s>>>(a);
    else k_attn<HD, 2><<<grid, 512, 0, s>>>(a);
    PV_HIP(hipGetLastError());
    k_attn_merge<NB, HD><<<dim3(rows, f.n_q_heads), 256, 0, s>>>(a, mp);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

// q (fp32, rotated) -> xop_o; part = scratch of pv_attn_part_floats floats
int pv_mat_attention(pv_cache *c, int layer, int rows, float *part, uint16_t *xop_o, hipStream_t s)
{
    const pv_model_config &f = c->m->cfg;
    attn_args a;
    a.st = c->ws.state; a.page_table = c->ws.page_table; a.q = c->ws.q; a.pool = (const uint16_t *)c->d_pool;
    a.geom = pv_geom(c); a.layer = layer; a.n_q_heads = f.n_q_heads; a.group = f.n_q_heads / f.n_kv_heads;
    a.max_chunks = (c->max_tokens + 255) / 256;
    a.scale = 1.0f / sqrtf((float)f.head_dim);
    const int mp_cap = (a.group * c->rows_cap + 31) / 32;
    a.part_o = part;
    a.part_ml = part + (size_t)f.n_kv_heads * mp_cap * a.max_chunks * 32 * f.head_dim;
    a.xop_o = xop_o;
    const bool nb1 = rows <= 8;
    switch (f.head_dim) {
    case 32: return nb1 ? launch<1, 32>(c, a, rows, s) : launch<2, 32>(c, a, rows, s);
    case 64: return nb1 ? launch<1, 64>(c, a, rows, s) : launch<2, 64>(c, a, rows, s);
    case 128: return nb1 ? launch<1, 128>(c, a, rows, s) : launch<2, 128>(c, a, rows, s);
    default: pv_set_error("matrix path: unsupported head_dim %d", f.head_dim); return PV_EINVAL;
    }
}
