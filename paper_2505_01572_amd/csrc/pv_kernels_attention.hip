// Causal grouped-query attention over the paged bf16 KV cache on the matrix cores.
//
// Work unit: one workgroup = (kv head, chunk of 256 keys, group of <= 32 query rows).  The
// query rows of a kv head are its `group` query heads x gamma block rows, packed densely
// (row m = head_in_group * gamma + j).  Each of the 4 wavefronts takes 64 keys in two steps of
// 32; the four partial results are merged through LDS in wave order and written as one
// partial (max, sum, output) per chunk; a small merge kernel combines the chunks and writes
// the attention output directly as the output projection's split-bf16 operand.
//
// Everything is computed transposed so that no register shuffling is needed:
//   S^T (keys x rows) = K (keys x hd) * Q^T (hd x rows)      A = K tile, B = Q^T
//   O^T (hd x rows)   = V^T (hd x keys) * P^T (keys x rows)   A = V^T tile, B = P^T
// A 16-key page group stored as [hd/32][lane][8] is exactly the A operand of the first
// product.  The accumulator of S^T holds, per lane, 4 consecutive keys of row lane%16 — and
// that is, for two key groups side by side, the B operand of the second product when the 32
// keys of a step are taken in the order (group0 keys 4g..4g+3, group1 keys 4g..4g+3); V^T is
// read in that same order (8-byte loads from the [hd][16] page layout).  Softmax statistics
// of row lane%16 then sit in the same lane as that row's output accumulators.
//
// Q and P are carried as bf16 hi + lo pairs (two MFMAs each), K and V are the stored bf16.
// The causal part only touches keys >= len: key p is visible to block row j iff p <= len + j.
#include "pv_matrix_common.h"

struct attn_args {
    const pv_dev_state *st;
    const int32_t *page_table;
    const float *q;             // [rows][n_q_heads][hd], rotary already applied
    const uint16_t *pool;
    pv_kv_geom geom;
    int layer, n_q_heads, group, max_chunks;
    float scale;
    float *part_o;              // [n_kv_heads][MP][max_chunks][32][hd]
    float *part_ml;             // [n_kv_heads][MP][max_chunks][32][2]  (max, sum)
    uint16_t *xop_o;            // merge output: operand of the output projection, K = n_q_heads*hd
};

__device__ inline void split8(const float v[8], uint4 &hi, uint4 &lo)
{
    uint32_t h[4], l[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const uint16_t h0 = pv_f32_to_bf16(v[2 * i]), h1 = pv_f32_to_bf16(v[2 * i + 1]);
        const uint16_t l0 = pv_f32_to_bf16(v[2 * i] - pv_bf16_to_f32(h0)), l1 = pv_f32_to_bf16(v[2 * i + 1] - pv_bf16_to_f32(h1));
        h[i] = h0 | ((uint32_t)h1 << 16); l[i] = l0 | ((uint32_t)l1 << 16);
    }
    hi = make_uint4(h[0], h[1], h[2], h[3]); lo = make_uint4(l[0], l[1], l[2], l[3]);
}

template <int HD, int R>
__global__ void __launch_bounds__(256)
k_attn(const attn_args a)
{
    constexpr int KS = HD / 32, ET = HD / 16, OS = HD + 1;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, jl = lane & 15, g = lane >> 4;
    const int c = blockIdx.x, kvh = blockIdx.y, mp = blockIdx.z;
    const int len = a.st->len, gamma = a.st->gamma, nkeys = len + gamma;
    if (c * 256 >= nkeys) return;
    const int nrows = a.group * gamma;
    const pv_kv_geom &gm = a.geom;
    const int sub_shift = gm.page_shift - 4, sub_mask = (1 << sub_shift) - 1;

    // Q^T operands of this lane's rows (row = lane%16 of each 16-row tile), hi and lo
    uint4 qh[R][KS], ql[R][KS];
    int lim[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int m = mp * 32 + rt * 16 + jl;
        const bool live = m < nrows;
        const int al = live ? m / gamma : 0, j = live ? m - al * gamma : 0;
        lim[rt] = live ? len + j : -1;
        const float *qp = a.q + ((size_t)j * a.n_q_heads + kvh * a.group + al) * HD + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            float v[8];
            if (live) {
                const float4 x0 = *(const float4 *)(qp + ks * 32), x1 = *(const float4 *)(qp + ks * 32 + 4);
                v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w; v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
            } else {
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = 0.f;
            }
            split8(v, qh[rt][ks], ql[rt][ks]);
        }
    }

    f32x4 O[R][ET];
    float mrow[R], lrow[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        mrow[rt] = -INFINITY; lrow[rt] = 0.f;
#pragma unroll
        for (int et = 0; et < ET; ++et) O[rt][et] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }

    const int k0 = c * 256 + wave * 64;
    for (int step = 0; step < 2; ++step) {
        const int p0 = k0 + step * 32;
        if (p0 >= nkeys) break;
        // two groups of 16 keys; the second may lie past the end: read the first again, it is masked
        const int g0 = p0 >> 4, g1 = (p0 + 16 < nkeys) ? g0 + 1 : g0;
        const uint16_t *kb[2], *vb[2];
        {
            const int ph0 = a.page_table[g0 >> sub_shift], ph1 = a.page_table[g1 >> sub_shift];
            kb[0] = a.pool + pv_kv_block(gm, a.layer, ph0, kvh, 0) + (size_t)(g0 & sub_mask) * 16 * HD;
            kb[1] = a.pool + pv_kv_block(gm, a.layer, ph1, kvh, 0) + (size_t)(g1 & sub_mask) * 16 * HD;
            vb[0] = a.pool + pv_kv_block(gm, a.layer, ph0, kvh, 1) + (size_t)(g0 & sub_mask) * 16 * HD;
            vb[1] = a.pool + pv_kv_block(gm, a.layer, ph1, kvh, 1) + (size_t)(g1 & sub_mask) * 16 * HD;
        }
        uint4 kt[2][KS];
        uint2 vt[2][ET];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) kt[t][ks] = ((const uint4 *)kb[t])[ks * 64 + lane];
#pragma unroll
            for (int et = 0; et < ET; ++et) vt[t][et] = *(const uint2 *)(vb[t] + (size_t)(et * 16 + jl) * 16 + 4 * g);
        }
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s0 = mfma16(kt[0][ks], qh[rt][ks], s0); s0 = mfma16(kt[0][ks], ql[rt][ks], s0);
                s1 = mfma16(kt[1][ks], qh[rt][ks], s1); s1 = mfma16(kt[1][ks], ql[rt][ks], s1);
            }
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int pa = p0 + 4 * g + r, pb = pa + 16;
                sv[r] = (pa <= lim[rt]) ? s0[r] * a.scale : -INFINITY;
                sv[4 + r] = (pb <= lim[rt]) ? s1[r] * a.scale : -INFINITY;
                mx = fmaxf(mx, fmaxf(sv[r], sv[4 + r]));
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(mrow[rt], mx);
            const bool none = m_new == -INFINITY;              // no visible key for this row so far
            const float resc = none ? 1.f : expf(mrow[rt] - m_new);
            float pr[8], ps = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) { pr[i] = none ? 0.f : expf(sv[i] - m_new); ps += pr[i]; }
            lrow[rt] = lrow[rt] * resc + ps;
            mrow[rt] = m_new;
            uint4 ph, pl;
            split8(pr, ph, pl);
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                f32x4 o = O[rt][et];
                o[0] *= resc; o[1] *= resc; o[2] *= resc; o[3] *= resc;
                const uint4 va = make_uint4(vt[0][et].x, vt[0][et].y, vt[1][et].x, vt[1][et].y);
                o = mfma16(va, ph, o);
                o = mfma16(va, pl, o);
                O[rt][et] = o;
            }
        }
    }

    // merge the four waves (fixed order) and write the chunk's partial
    __shared__ float sh_m[4][R * 16], sh_M[R * 16], sh_l[R * 16], sh_o[R * 16][OS];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        lrow[rt] += __shfl_xor(lrow[rt], 16, 64);
        lrow[rt] += __shfl_xor(lrow[rt], 32, 64);
        if (g == 0) sh_m[wave][rt * 16 + jl] = mrow[rt];
    }
    __syncthreads();
    float f[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int row = rt * 16 + jl;
        const float M = fmaxf(fmaxf(sh_m[0][row], sh_m[1][row]), fmaxf(sh_m[2][row], sh_m[3][row]));
        f[rt] = (mrow[rt] == -INFINITY) ? 0.f : expf(mrow[rt] - M);
        if (wave == 0 && g == 0) sh_M[row] = M;
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                const int row = rt * 16 + jl;
#pragma unroll
                for (int et = 0; et < ET; ++et)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float val = O[rt][et][r] * f[rt];
                        float *dst = &sh_o[row][et * 16 + 4 * g + r];
                        *dst = (w == 0) ? val : *dst + val;
                    }
                if (g == 0) sh_l[row] = (w == 0) ? lrow[rt] * f[rt] : sh_l[row] + lrow[rt] * f[rt];
            }
        }
        __syncthreads();
    }
    const size_t unit = ((size_t)kvh * gridDim.z + mp) * a.max_chunks + c;
    float *po = a.part_o + unit * 32 * HD;
    for (int i = threadIdx.x; i < R * 16 * HD; i += 256) po[i] = sh_o[i / HD][i % HD];
    if (threadIdx.x < R * 16) {
        float *pm = a.part_ml + (unit * 32 + threadIdx.x) * 2;
        pm[0] = sh_M[threadIdx.x]; pm[1] = sh_l[threadIdx.x];
    }
}

// Combine the chunk partials of one (block row, query head) and emit the operand of the
// output projection.  One thread per 4 consecutive features.
template <int NB, int HD>
__global__ void __launch_bounds__(64)
k_attn_merge(const attn_args a, int mp_count)
{
    const int j = blockIdx.x, aq = blockIdx.y, gamma = a.st->gamma;
    if (j >= gamma) return;
    const int kvh = aq / a.group, al = aq - kvh * a.group, m = al * gamma + j, mp = m >> 5, row = m & 31;
    const int nchunks = (a.st->len + gamma + 255) >> 8;
    const size_t unit0 = ((size_t)kvh * mp_count + mp) * a.max_chunks;
    float M = -INFINITY;
    for (int c = 0; c < nchunks; ++c) M = fmaxf(M, a.part_ml[((unit0 + c) * 32 + row) * 2]);
    const int t = threadIdx.x;
    if (t >= HD / 4) return;
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, L = 0.f;
    for (int c = 0; c < nchunks; ++c) {
        const float *pm = a.part_ml + ((unit0 + c) * 32 + row) * 2;
        const float w = (pm[0] == -INFINITY) ? 0.f : expf(pm[0] - M);
        L += pm[1] * w;
        const float4 o = *(const float4 *)(a.part_o + ((unit0 + c) * 32 + row) * HD + 4 * t);
        acc[0] += w * o.x; acc[1] += w * o.y; acc[2] += w * o.z; acc[3] += w * o.w;
    }
    const float inv = 1.0f / L;
    const float y[4] = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
    store_operand4<NB>(a.xop_o, a.n_q_heads * HD, j, aq * HD + 4 * t, y);
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
    if (nrows <= 16) k_attn<HD, 1><<<grid, 256, 0, s>>>(a);
    else k_attn<HD, 2><<<grid, 256, 0, s>>>(a);
    PV_HIP(hipGetLastError());
    k_attn_merge<NB, HD><<<dim3(rows, f.n_q_heads), 64, 0, s>>>(a, mp);
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
