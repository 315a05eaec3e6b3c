// Causal grouped-query attention over the paged bf16 KV cache on the matrix cores.
//
// Work unit: one workgroup = (kv head, chunk of 256 keys, group of <= 32 query rows).  The
// query rows of a kv head are its `group` query heads x gamma block rows, packed densely
// (row m = head_in_group * gamma + j).  Each of the 8 wavefronts takes 32 keys; the eight
// partial results are merged through LDS in a fixed order and written as one partial (max,
// sum, output) per chunk; a small merge kernel combines the chunks and writes the attention
// output directly as the output projection's split-bf16 operand.
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
#pragma once
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

template <int HD, int R, int HALVES>
__host__ __device__ constexpr int attn_smem_floats() { return 8 * R * 16 + R * 16 + HALVES * R * 16 + HALVES * R * 16 * (HD + 1); }

// One (kv head, 256-key chunk, 32-row group) unit, executed by 8 wavefronts (threads 0..511 of
// the calling workgroup; every thread of those 8 waves must call it).  HALVES = 2 merges the
// waves in two side-by-side sequences (needs twice the LDS), HALVES = 1 in one sequence.
// smem: attn_smem_floats<HD, R, HALVES>() floats of LDS.
template <int HD, int R, int HALVES>
__device__ inline void attn_chunk(const attn_args &a, int c, int kvh, int mp, int n_mp, float *smem)
{
    constexpr int KS = HD / 32, ET = HD / 16, OS = HD + 1;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, jl = lane & 15, g = lane >> 4;
    const int len = a.st->len, gamma = a.st->gamma, nkeys = len + gamma;
    if (c * 256 >= nkeys) return;
    const int nrows = a.group * gamma;
    const pv_kv_geom &gm = a.geom;
    const int sub_shift = gm.page_shift - 4, sub_mask = (1 << sub_shift) - 1;

    // this wave's 32 keys: two groups of 16; a group past the end re-reads the first one (it is masked)
    const int p0 = c * 256 + wave * 32;
    const bool has_keys = p0 < nkeys;
    uint4 kt[2][KS];
    uint2 vt[2][ET];
    if (has_keys) {
        const int g0 = p0 >> 4, g1 = (p0 + 16 < nkeys) ? g0 + 1 : g0;
        const int ph0 = a.page_table[g0 >> sub_shift], ph1 = a.page_table[g1 >> sub_shift];
        const uint16_t *kb0 = a.pool + pv_kv_block(gm, a.layer, ph0, kvh, 0) + (size_t)(g0 & sub_mask) * 16 * HD;
        const uint16_t *kb1 = a.pool + pv_kv_block(gm, a.layer, ph1, kvh, 0) + (size_t)(g1 & sub_mask) * 16 * HD;
        const uint16_t *vb0 = a.pool + pv_kv_block(gm, a.layer, ph0, kvh, 1) + (size_t)(g0 & sub_mask) * 16 * HD;
        const uint16_t *vb1 = a.pool + pv_kv_block(gm, a.layer, ph1, kvh, 1) + (size_t)(g1 & sub_mask) * 16 * HD;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) { kt[0][ks] = ((const uint4 *)kb0)[ks * 64 + lane]; kt[1][ks] = ((const uint4 *)kb1)[ks * 64 + lane]; }
#pragma unroll
        for (int et = 0; et < ET; ++et) {
            vt[0][et] = *(const uint2 *)(vb0 + (size_t)(et * 16 + jl) * 16 + 4 * g);
            vt[1][et] = *(const uint2 *)(vb1 + (size_t)(et * 16 + jl) * 16 + 4 * g);
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

    if (has_keys) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt) {
            // Q^T operand of this lane's row (row = lane%16 of the 16-row tile), hi and lo
            const int m = mp * 32 + rt * 16 + jl;
            const bool live = m < nrows;
            const int al = live ? m / gamma : 0, j = live ? m - al * gamma : 0;
            const int lim = live ? len + j : -1;
            const float *qp = a.q + ((size_t)j * a.n_q_heads + kvh * a.group + al) * HD + g * 8;
            f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                float v[8];
                const float4 x0 = *(const float4 *)(qp + ks * 32), x1 = *(const float4 *)(qp + ks * 32 + 4);
                v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w; v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
                if (!live) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = 0.f;
                }
                uint4 qh, ql;
                split8(v, qh, ql);
                s0 = mfma16(kt[0][ks], qh, s0); s0 = mfma16(kt[0][ks], ql, s0);
                s1 = mfma16(kt[1][ks], qh, s1); s1 = mfma16(kt[1][ks], ql, s1);
            }
            float sv[8];
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int pa = p0 + 4 * g + r, pb = pa + 16;
                sv[r] = (pa <= lim) ? s0[r] * a.scale : -INFINITY;
                sv[4 + r] = (pb <= lim) ? s1[r] * a.scale : -INFINITY;
                mx = fmaxf(mx, fmaxf(sv[r], sv[4 + r]));
            }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const bool none = mx == -INFINITY;                 // no visible key for this row here
            float pr[8], ps = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) { pr[i] = none ? 0.f : expf(sv[i] - mx); ps += pr[i]; }
            ps += __shfl_xor(ps, 16, 64);
            ps += __shfl_xor(ps, 32, 64);
            lrow[rt] = ps; mrow[rt] = mx;
            uint4 ph, pl;
            split8(pr, ph, pl);
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                const uint4 va = make_uint4(vt[0][et].x, vt[0][et].y, vt[1][et].x, vt[1][et].y);
                f32x4 o = {0.f, 0.f, 0.f, 0.f};
                o = mfma16(va, ph, o);
                o = mfma16(va, pl, o);
                O[rt][et] = o;
            }
        }
    }

    // merge the eight waves in a fixed order: waves 0..3 into buffer 0, waves 4..7 into buffer 1
    // (both sequences run side by side), then buffer 0 + buffer 1 while writing the partial
    float (*sh_m)[R * 16] = (float (*)[R * 16])smem;                              // [8][R*16]
    float *sh_M = smem + 8 * R * 16;                                              // [R*16]
    float (*sh_l)[R * 16] = (float (*)[R * 16])(sh_M + R * 16);                   // [HALVES][R*16]
    float (*sh_o)[R * 16][OS] = (float (*)[R * 16][OS])(sh_M + R * 16 + HALVES * R * 16);   // [HALVES][R*16][OS]
    if (g == 0) {
#pragma unroll
        for (int rt = 0; rt < R; ++rt) sh_m[wave][rt * 16 + jl] = mrow[rt];
    }
    __syncthreads();
    float f[R];
#pragma unroll
    for (int rt = 0; rt < R; ++rt) {
        const int row = rt * 16 + jl;
        float M = sh_m[0][row];
#pragma unroll
        for (int w = 1; w < 8; ++w) M = fmaxf(M, sh_m[w][row]);
        f[rt] = (mrow[rt] == -INFINITY) ? 0.f : expf(mrow[rt] - M);
        if (wave == 0 && g == 0) sh_M[row] = M;
    }
    const int half = (HALVES == 2) ? wave >> 2 : 0, wq = (HALVES == 2) ? wave & 3 : wave;
    for (int w = 0; w < 8 / HALVES; ++w) {
        if (wq == w) {
#pragma unroll
            for (int rt = 0; rt < R; ++rt) {
                const int row = rt * 16 + jl;
#pragma unroll
                for (int et = 0; et < ET; ++et)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float val = O[rt][et][r] * f[rt];
                        float *dst = &sh_o[half][row][et * 16 + 4 * g + r];
                        *dst = (w == 0) ? val : *dst + val;
                    }
                if (g == 0) sh_l[half][row] = (w == 0) ? lrow[rt] * f[rt] : sh_l[half][row] + lrow[rt] * f[rt];
            }
        }
        __syncthreads();
    }
    const size_t unit = ((size_t)kvh * n_mp + mp) * a.max_chunks + c;
    float *po = a.part_o + unit * 32 * HD;
    for (int i = threadIdx.x; i < R * 16 * HD; i += 512) po[i] = (HALVES == 2) ? sh_o[0][i / HD][i % HD] + sh_o[HALVES - 1][i / HD][i % HD] : sh_o[0][i / HD][i % HD];
    if (threadIdx.x < R * 16) {
        float *pm = a.part_ml + (unit * 32 + threadIdx.x) * 2;
        pm[0] = sh_M[threadIdx.x]; pm[1] = (HALVES == 2) ? sh_l[0][threadIdx.x] + sh_l[HALVES - 1][threadIdx.x] : sh_l[0][threadIdx.x];
    }
}

// Combine the chunk partials of one (block row, query head) and emit the operand of the
// output projection.  One thread per 4 consecutive features.
// (block row j, query head aq) unit, executed by NT threads (tid = 0..NT-1, all must call).
// smem: NT + (NT / (HD/4)) * (HD/4) * 5 floats.
template <int NB, int HD, int NT>
__device__ inline void attn_merge_unit(const attn_args &a, int j, int aq, int mp_count, int tid, float *smem)
{
    constexpr int TPC = HD / 4;            // threads per chunk: 4 consecutive features each
    constexpr int NG = NT / TPC;           // chunk groups working side by side
    const int gamma = a.st->gamma;
    const int kvh = aq / a.group, al = aq - kvh * a.group, m = al * gamma + j, mp = m >> 5, row = m & 31;
    const int nchunks = (a.st->len + gamma + 255) >> 8;
    const size_t unit0 = ((size_t)kvh * mp_count + mp) * a.max_chunks;
    float *sh_m = smem;                                              // [NT]
    float (*sh_acc)[TPC][5] = (float (*)[TPC][5])(smem + NT);        // [NG][TPC][5]
    // global max over chunks (each thread looks at chunks t, t+256, ...)
    float M = -INFINITY;
    for (int c = tid; c < nchunks; c += NT) M = fmaxf(M, a.part_ml[((unit0 + c) * 32 + row) * 2]);
    sh_m[tid] = M;
    __syncthreads();
    for (int s2 = NT / 2; s2 > 0; s2 >>= 1) {
        if ((int)tid < s2) sh_m[tid] = fmaxf(sh_m[tid], sh_m[tid + s2]);
        __syncthreads();
    }
    M = sh_m[0];
    const int t = tid % TPC, cg = tid / TPC;
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, L = 0.f;
    for (int c = cg; c < nchunks; c += NG) {
        const float *pm = a.part_ml + ((unit0 + c) * 32 + row) * 2;
        const float w = (pm[0] == -INFINITY) ? 0.f : expf(pm[0] - M);
        L += pm[1] * w;
        const float4 o = *(const float4 *)(a.part_o + ((unit0 + c) * 32 + row) * HD + 4 * t);
        acc[0] += w * o.x; acc[1] += w * o.y; acc[2] += w * o.z; acc[3] += w * o.w;
    }
    sh_acc[cg][t][0] = acc[0]; sh_acc[cg][t][1] = acc[1]; sh_acc[cg][t][2] = acc[2]; sh_acc[cg][t][3] = acc[3]; sh_acc[cg][t][4] = L;
    __syncthreads();
    if (cg != 0) return;
    for (int o2 = 1; o2 < NG; ++o2) {
        acc[0] += sh_acc[o2][t][0]; acc[1] += sh_acc[o2][t][1]; acc[2] += sh_acc[o2][t][2]; acc[3] += sh_acc[o2][t][3]; L += sh_acc[o2][t][4];
    }
    const float inv = 1.0f / L;
    const float y[4] = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
    store_operand4<NB>(a.xop_o, a.n_q_heads * HD, j, aq * HD + 4 * t, y);
}

