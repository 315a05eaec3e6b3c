// Causal grouped-query attention over the paged bf16 KV cache on the matrix cores.
//
// Work unit: one workgroup of 8 wavefronts = (kv head, chunk of keys, group of <= 32 query
// rows).  The query rows of a kv head are its `group` query heads x gamma block rows, packed
// densely (row m = head_in_group * gamma + j).  Two shapes of the unit:
//   TILES = 1: up to 16 rows, 256 keys; every wave takes 32 keys of the one 16-row tile;
//   TILES = 2: 17..32 rows, 128 keys; wave w takes row tile w / 4 and 32 keys (w % 4).
// Either way a wave makes one pass.  The waves of a row tile are merged through LDS (every
// wave writes its rescaled partial, then all threads add them in wave order) into one partial
// (max, sum, output) per chunk; a small merge kernel combines the chunks and writes the
// attention output directly as the output projection's split-bf16 operand.
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
// Softmax weights use the hardware exponential (__expf, relative error ~1e-6 at these
// arguments): they are rounded to 16 mantissa bits for the second product anyway.
// Q arrives already split (the QKV projection's epilogue writes the two bf16 arrays).
// The causal part only touches keys >= len: block row j sees the block slots its mask names (a chain:
// keys up to len + j; a draft tree: its ancestors' slots and its own).
#pragma once
#include "pv_matrix_common.h"

struct attn_args {
    const pv_dev_state *st;
    const int32_t *page_table;
    const uint16_t *q_hi, *q_lo; // [rows][n_q_heads][hd] each, rotary already applied: q = hi + lo
    const uint16_t *pool;
    pv_kv_geom geom;
    int layer, n_q_heads, group, max_chunks;
    int chunk_shift;            // log2 of the keys per chunk of the partials (8 with one row tile, 7 with two)
    float scale;
    float *part_o;              // [n_kv_heads][MP][max_chunks][32][hd]
    float *part_ml;             // [n_kv_heads][MP][max_chunks][32][2]  (max, sum)
    uint16_t *xop_o;            // merge output: operand of the output projection, K = n_q_heads*hd
    int n_pages;                // entries of the page table
    int lo_off;                 // column offset of the lo halves in the output operand's tiles (packed rows)
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

template <int HD>
__host__ __device__ constexpr int attn_smem_floats() { return 8 * 16 * (HD + 4) + 2 * 8 * 16; }

// One (kv head, chunk, 32-row group) unit, executed by the 8 wavefronts of the workgroup (all
// 512 threads must call).  TILES as above; chunk c covers keys c * (256 / TILES) ... .
// smem: attn_smem_floats<HD>() floats of LDS (more than 64 KiB for HD = 128: dynamic).
template <int HD, int TILES>
__device__ inline void attn_chunk(const attn_args &a, int c, int kvh, int z, int n_units, float *smem)
{
    constexpr int KS = HD / 32, ET = HD / 16, OS = HD + 4, NWM = 8 / TILES, CK = 256 / TILES;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, jl = lane & 15, g = lane >> 4;
    const int rt = wave / NWM, kq = wave % NWM;
    pv_kv_geom gm = a.geom;
    const int sub_shift = gm.page_shift - 4, sub_mask = (1 << sub_shift) - 1;
    // this wave's 32 keys: two groups of 16.  Which pages they sit in does not depend on the cache
    // length, so the page-table entries are fetched beside the length, not behind it (an entry past
    // the table's end is clamped; such keys are past the length as well and never used).
    const int p0 = c * CK + kq * 32;
    int ph0 = a.page_table[min((p0 >> 4) >> sub_shift, a.n_pages - 1)], ph1g = a.page_table[min(((p0 >> 4) + 1) >> sub_shift, a.n_pages - 1)];
    const int nseq = a.st->blk.n_seq;
    int len = a.st->len, gamma = a.st->gamma, row0 = 0, mp = z;
    const uint16_t *pool = a.pool;
    if (nseq > 1) {
        // batched step: unit z belongs to the sequence with the largest unit0 <= z; its rows, length and pages
        int sidx = 0;
        for (int k = 1; k < nseq; ++k) if (z >= a.st->blk.seq[k].unit0) sidx = k;
        const pv_seq_ref &sq = a.st->blk.seq[sidx];
        len = sq.st->len; gamma = sq.gamma; row0 = sq.row0; mp = z - sq.unit0;
        pool = (const uint16_t *)sq.pool; gm.n_pages = sq.n_pages;
        ph0 = sq.page_table[min((p0 >> 4) >> sub_shift, sq.n_pages - 1)]; ph1g = sq.page_table[min(((p0 >> 4) + 1) >> sub_shift, sq.n_pages - 1)];
    }
    const int nkeys = len + gamma;
    if (c * CK >= nkeys) return;
    const int nrows = a.group * gamma;
    if (mp * 32 >= nrows) return;                      // (a unit beyond the sequence's rows: the grid is sized for the largest)
    const bool has_keys = p0 < nkeys;
    // this lane's query row: row lane%16 of the wave's 16-row tile
    const int m = mp * 32 + rt * 16 + jl;
    const bool live = m < nrows;
    const int al = live ? m / gamma : 0, j = live ? m - al * gamma : 0;
    // which keys the row may see: every committed position, and of the block's own slots (len + q) those its
    // mask names (a chain: up to its own; a draft tree: its ancestors and itself); a dead lane sees nothing
    const uint64_t vmask = live ? a.st->rowmask[row0 + j] : 0ull;
    auto visible = [&](int p) { const int q = p - len; return live && (q < 0 || (q < 64 && ((vmask >> q) & 1ull))); };
    uint4 kt[2][KS], qh[KS], ql[KS];
    uint2 vt[2][ET];
    if (has_keys) {
        // a second group past the end re-reads the first one (it is masked)
        const bool two = p0 + 16 < nkeys;
        const int g0 = p0 >> 4, g1 = two ? g0 + 1 : g0;
        const int ph1 = two ? ph1g : ph0;
        // a dead lane reads row 0 of the first head: its scores are masked below
        const size_t qoff = ((size_t)(row0 + j) * a.n_q_heads + kvh * a.group + al) * HD + g * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qh[ks] = *(const uint4 *)(a.q_hi + qoff + ks * 32);
            ql[ks] = *(const uint4 *)(a.q_lo + qoff + ks * 32);
        }
        const uint16_t *kb0 = pool + pv_kv_block(gm, a.layer, ph0, kvh, 0) + (size_t)(g0 & sub_mask) * 16 * HD;
        const uint16_t *kb1 = pool + pv_kv_block(gm, a.layer, ph1, kvh, 0) + (size_t)(g1 & sub_mask) * 16 * HD;
        const uint16_t *vb0 = pool + pv_kv_block(gm, a.layer, ph0, kvh, 1) + (size_t)(g0 & sub_mask) * 16 * HD;
        const uint16_t *vb1 = pool + pv_kv_block(gm, a.layer, ph1, kvh, 1) + (size_t)(g1 & sub_mask) * 16 * HD;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) { kt[0][ks] = ((const uint4 *)kb0)[ks * 64 + lane]; kt[1][ks] = ((const uint4 *)kb1)[ks * 64 + lane]; }
#pragma unroll
        for (int et = 0; et < ET; ++et) {
            vt[0][et] = *(const uint2 *)(vb0 + (size_t)(et * 16 + jl) * 16 + 4 * g);
            vt[1][et] = *(const uint2 *)(vb1 + (size_t)(et * 16 + jl) * 16 + 4 * g);
        }
    }
    // every load above is in flight before the first use: one memory round trip, not one per operand
    asm volatile("" ::: "memory");

    f32x4 O[ET];
    float mrow = -INFINITY, lrow = 0.f;
#pragma unroll
    for (int et = 0; et < ET; ++et) O[et] = (f32x4){0.f, 0.f, 0.f, 0.f};

    if (has_keys) {
        f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            s0 = mfma16(kt[0][ks], qh[ks], s0); s1 = mfma16(kt[1][ks], qh[ks], s1);
            s0 = mfma16(kt[0][ks], ql[ks], s0); s1 = mfma16(kt[1][ks], ql[ks], s1);
        }
        float sv[8];
        float mx = -INFINITY;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int pa = p0 + 4 * g + r, pb = pa + 16;
            sv[r] = visible(pa) ? s0[r] * a.scale : -INFINITY;
            sv[4 + r] = visible(pb) ? s1[r] * a.scale : -INFINITY;
            mx = fmaxf(mx, fmaxf(sv[r], sv[4 + r]));
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const bool none = mx == -INFINITY;                 // no visible key for this row here
        float pr[8], ps = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) { pr[i] = none ? 0.f : __expf(sv[i] - mx); ps += pr[i]; }
        ps += __shfl_xor(ps, 16, 64);
        ps += __shfl_xor(ps, 32, 64);
        lrow = ps; mrow = mx;
        uint4 ph, pl;
        split8(pr, ph, pl);
#pragma unroll
        for (int et = 0; et < ET; ++et) {
            const uint4 va = make_uint4(vt[0][et].x, vt[0][et].y, vt[1][et].x, vt[1][et].y);
            f32x4 o = {0.f, 0.f, 0.f, 0.f};
            o = mfma16(va, ph, o);
            o = mfma16(va, pl, o);
            O[et] = o;
        }
    }

    // merge the NWM waves of each row tile: every wave parks its partial, rescaled to the
    // tile's common maximum, in LDS; then all threads add the NWM partials in wave order
    float (*sh_m)[16] = (float (*)[16])smem;                                  // [8][16]
    float (*sh_l)[16] = (float (*)[16])(smem + 8 * 16);                       // [8][16]
    float (*sh_o)[16][OS] = (float (*)[16][OS])(smem + 2 * 8 * 16);           // [8][16][OS]
    if (g == 0) sh_m[wave][jl] = mrow;
    __syncthreads();
    float M = sh_m[rt * NWM][jl];
#pragma unroll
    for (int w = 1; w < NWM; ++w) M = fmaxf(M, sh_m[rt * NWM + w][jl]);
    const float f = (mrow == -INFINITY) ? 0.f : __expf(mrow - M);
#pragma unroll
    for (int et = 0; et < ET; ++et)
        *(float4 *)&sh_o[wave][jl][et * 16 + 4 * g] = make_float4(O[et][0] * f, O[et][1] * f, O[et][2] * f, O[et][3] * f);
    if (g == 0) sh_l[wave][jl] = lrow * f;
    __syncthreads();
    const size_t unit = ((size_t)kvh * n_units + z) * a.max_chunks + c;
    float *po = a.part_o + unit * 32 * HD;
    for (int i = threadIdx.x; i < TILES * 16 * (HD / 4); i += 512) {
        const int row = i / (HD / 4), c4 = i - row * (HD / 4), t = row >> 4, r = row & 15;
        float4 acc = *(const float4 *)&sh_o[t * NWM][r][4 * c4];
#pragma unroll
        for (int w = 1; w < NWM; ++w) {
            const float4 v = *(const float4 *)&sh_o[t * NWM + w][r][4 * c4];
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
        *(float4 *)(po + (size_t)row * HD + 4 * c4) = acc;
    }
    if (threadIdx.x < TILES * 16) {
        const int t = threadIdx.x >> 4, r = threadIdx.x & 15;
        float Mr = sh_m[t * NWM][r], L = sh_l[t * NWM][r];
#pragma unroll
        for (int w = 1; w < NWM; ++w) { Mr = fmaxf(Mr, sh_m[t * NWM + w][r]); L += sh_l[t * NWM + w][r]; }
        float *pm = a.part_ml + (unit * 32 + threadIdx.x) * 2;
        pm[0] = Mr; pm[1] = L;
    }
}

// Combine the chunk partials of one (block row, query head) and emit the operand of the
// output projection.  One thread per 4 consecutive features.
// (block row j, query head aq) unit, executed by NT threads (tid = 0..NT-1, all must call).
// smem: NT + (NT / (HD/4)) * (HD/4) * 5 floats.
template <int NB, int HD, int NT>
__device__ inline void attn_merge_unit(const attn_args &a, int r, int aq, int n_units, int tid, float *smem)
{
    constexpr int TPC = HD / 4;            // threads per chunk: 4 consecutive features each
    constexpr int NG = NT / TPC;           // chunk groups working side by side
    // block row r: its sequence's rows, length and first unit (a plain step: the cache itself)
    const int nseq = a.st->blk.n_seq;
    int gamma = a.st->gamma, len = a.st->len, row0 = 0, unit_s = 0;
    if (nseq > 1) {
        const pv_seq_ref &sq = a.st->blk.seq[a.st->rowseq[r]];
        gamma = sq.gamma; len = sq.st->len; row0 = sq.row0; unit_s = sq.unit0;
    }
    const int j = r - row0;
    const int kvh = aq / a.group, al = aq - kvh * a.group, m = al * gamma + j, mp = m >> 5, row = m & 31;
    const int nchunks = (len + gamma + (1 << a.chunk_shift) - 1) >> a.chunk_shift;
    const size_t unit0 = ((size_t)kvh * n_units + unit_s + mp) * a.max_chunks;
    float *sh_m = smem;                                              // [NT]
    float (*sh_acc)[TPC][5] = (float (*)[TPC][5])(smem + NT);        // [NG][TPC][5]
    const int t = tid % TPC, cg = tid / TPC;
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, L = 0.f;
    if (nchunks <= 64) {
        // Up to 64 chunks: lane c of every wave holds chunk c's (max, sum); the global max, the
        // weights and the total come from wave shuffles (every wave redundantly, no barrier), and
        // the partial outputs are then fetched four chunks at a time with nothing depending on them.
        const int lane = tid & 63;
        float2 ml = make_float2(-INFINITY, 0.f);
        if (lane < nchunks) ml = *(const float2 *)(a.part_ml + ((unit0 + lane) * 32 + row) * 2);
        float M = ml.x;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) M = fmaxf(M, __shfl_xor(M, o, 64));
        const float wl = (ml.x == -INFINITY) ? 0.f : expf(ml.x - M);
        L = ml.y * wl;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) L += __shfl_xor(L, o, 64);
        for (int base = 0; base < nchunks; base += 4 * NG) {      // same trip count in every lane: the shuffles below need all lanes
            float4 o[4]; float w[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int c = base + cg + u * NG, cc = c < nchunks ? c : 0;
                o[u] = *(const float4 *)(a.part_o + ((unit0 + cc) * 32 + row) * HD + 4 * t);
                w[u] = __shfl(wl, cc, 64);
                if (c >= nchunks) w[u] = 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) { acc[0] += w[u] * o[u].x; acc[1] += w[u] * o[u].y; acc[2] += w[u] * o[u].z; acc[3] += w[u] * o[u].w; }
        }
        if (cg != 0) L = 0.f;                     // the total is added up over the chunk groups below: count it once
    } else {
        // many chunks: each thread looks at chunks tid, tid+NT, ... and a tree in LDS finishes the max
        float M = -INFINITY;
        for (int c = tid; c < nchunks; c += NT) M = fmaxf(M, a.part_ml[((unit0 + c) * 32 + row) * 2]);
        sh_m[tid] = M;
        __syncthreads();
        for (int s2 = NT / 2; s2 > 0; s2 >>= 1) {
            if ((int)tid < s2) sh_m[tid] = fmaxf(sh_m[tid], sh_m[tid + s2]);
            __syncthreads();
        }
        M = sh_m[0];
        for (int c = cg; c < nchunks; c += NG) {
            const float *pm = a.part_ml + ((unit0 + c) * 32 + row) * 2;
            const float w = (pm[0] == -INFINITY) ? 0.f : expf(pm[0] - M);
            L += pm[1] * w;
            const float4 o = *(const float4 *)(a.part_o + ((unit0 + c) * 32 + row) * HD + 4 * t);
            acc[0] += w * o.x; acc[1] += w * o.y; acc[2] += w * o.z; acc[3] += w * o.w;
        }
    }
    sh_acc[cg][t][0] = acc[0]; sh_acc[cg][t][1] = acc[1]; sh_acc[cg][t][2] = acc[2]; sh_acc[cg][t][3] = acc[3]; sh_acc[cg][t][4] = L;
    __syncthreads();
    if (cg != 0) return;
    for (int o2 = 1; o2 < NG; ++o2) {
        acc[0] += sh_acc[o2][t][0]; acc[1] += sh_acc[o2][t][1]; acc[2] += sh_acc[o2][t][2]; acc[3] += sh_acc[o2][t][3]; L += sh_acc[o2][t][4];
    }
    const float inv = 1.0f / L;
    const float y[4] = {acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv};
    store_operand4<NB>(a.xop_o, a.n_q_heads * HD, r, aq * HD + 4 * t, y, a.lo_off);
}

