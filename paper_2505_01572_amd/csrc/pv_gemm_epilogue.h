// Fused epilogues of the streaming GEMMs, shared by the packed-row kernel, the shared-tile kernel
// of the wide blocks and its finishing kernel.  An epilogue runs in one wavefront that holds the complete 16-feature x 16-column
// accumulator of a strip: lane l has features 4*(l/16)+r (r = 0..3) of column l%16.
#pragma once
#include "pv_matrix_common.h"

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };
#define PV_SEQ_TAG_SHIFT 26     // physical page numbers stay below 2^26; the bits above carry a row's sequence in a batched step

struct gemm_args {
    const uint4 *W;             // tiled region, strip-major
    const uint4 *xop;           // operand (hi [+ lo array behind it when NB == 2])
    int ktiles;                 // K / 32
    int interleave;             // K assignment of the waves (see k_gemm)
    int half_base;              // first of the strips that two workgroups share half and half (k_gemm<..., HF>)
    float *tile_part;           // scratch for the K-slice partial sums of k_gemm_tile
    int nstrips;                // strips of this GEMM (a workgroup may own several; the last one may be ragged)
    const pv_dev_state *st;
    int lo_off;                 // packed rows (NB == 1): column offset of the lo halves in operand tiles, 8, or 4 for blocks of at most 4 rows
    // RMSNorm scale of the input rows (QKV, SWIGLU, LMHEAD)
    const float *ssq; int ssq_parts; float inv_d, eps;
    // QKV
    uint16_t *q_hi, *q_lo; uint16_t *pool; const int32_t *page_table; const float2 *rope; pv_kv_geom geom;
    int layer, n_q_heads, q_strips, k_strips;
    // RESID
    float *x; const uint16_t *gain_next; float *ssq_out; uint16_t *xop_out; int d;
    // SWIGLU
    uint16_t *xop_act; int F;
    // LMHEAD
    float *logits; float *pmax_val; int32_t *pmax_idx; int vocab;
};

// Shared tail of everything that produces a new residual stream value: store x, the partial
// sum of squares of this 16-feature strip, and (gain * x) as the next GEMM's operand.
// Rows come in column tiles of 16 (ct = 0 .. ): row j = 16 * ct + lane % 16; the sums of
// squares are kept per tile as [ct][d/16 strips][16].
template <int NB>
__device__ inline void emit_x(int lane, int rows, int strip, int d, const float v[4], uint2 gain4,
                              float *x, float *ssq, uint16_t *xop, int ct, int lo_off)
{
    const int jl = lane & 15, j = ct * 16 + jl, g = lane >> 4, n = strip * 16 + 4 * g;
    const bool live = j < rows;
    if (live) *(float4 *)(x + (size_t)j * d + n) = make_float4(v[0], v[1], v[2], v[3]);
    float ss = live ? (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]) : 0.f;
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (lane < 16) ssq[((size_t)ct * (d >> 4) + strip) * 16 + jl] = ss;
    if (live) {
        const float y[4] = {v[0] * pv_bf16_to_f32((uint16_t)(gain4.x & 0xffffu)), v[1] * pv_bf16_to_f32((uint16_t)(gain4.x >> 16)),
                            v[2] * pv_bf16_to_f32((uint16_t)(gain4.y & 0xffffu)), v[3] * pv_bf16_to_f32((uint16_t)(gain4.y >> 16))};
        store_operand4<NB>(xop, d, j, n, y, lo_off);
    }
}

// Sum of squares of the input rows from the [parts][16] per-strip partial sums, first level,
// in two halves so that the caller can put its main loop between issue and use.  Thread `tid`
// of `nthreads` takes the float4 groups tid, tid+nthreads, ... (all loads independent: a serial
// chain of L2 round trips would cost more than the weight stream it sits beside).
template <int N = 2> struct ssq_loads { float4 v[N]; };   // N float4 groups per thread go out at once

template <int N>
__device__ inline void ssq_issue(const float *ssq, int parts, int tid, int nthreads, ssq_loads<N> &L)
{
    const float4 *q = (const float4 *)ssq;
    const int n4 = parts * 4;
#pragma unroll
    for (int u = 0; u < N; ++u) { const int i = tid + u * nthreads; L.v[u] = q[i < n4 ? i : 0]; }   // no branch: masked in ssq_finish
}

// Second half: add up (plus any groups beyond the first N per thread), then combine the lanes
// of the wave that hold the same rows (equal lane % 4).  On return lanes 0..3 hold the wave's
// sums for rows 4*lane .. 4*lane+3.
template <int N>
__device__ inline float4 ssq_finish(const float *ssq, int parts, int tid, int nthreads, const ssq_loads<N> &L)
{
    const float4 *q = (const float4 *)ssq;
    const int n4 = parts * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int u = 0; u < N; ++u) {
        if (tid + u * nthreads < n4) { s.x += L.v[u].x; s.y += L.v[u].y; s.z += L.v[u].z; s.w += L.v[u].w; }
    }
    for (int i = tid + N * nthreads; i < n4; i += nthreads) { const float4 v = q[i]; s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w; }
#pragma unroll
    for (int o = 4; o <= 32; o <<= 1) {
        s.x += __shfl_xor(s.x, o, 64); s.y += __shfl_xor(s.y, o, 64); s.z += __shfl_xor(s.z, o, 64); s.w += __shfl_xor(s.w, o, 64);
    }
    return s;
}

// What an epilogue needs from memory (rj is filled in after the reduction from the waves' sums
// of squares).  The owner wave fetches it while its first weight batch is in flight and parks it
// in LDS, so that after the reduction only arithmetic and stores remain.
struct epi_pre {
    float rj;
    int rows, pos, phys;        // phys: physical page of the row's position; bits 26.. = 1 + the row's sequence in a batched step (0: the cache itself)
    float4 xo;
    uint2 gn;
    float2 cs[4];
};

template <int EPI>
__device__ inline void epi_prefetch(const gemm_args &a, int strip, int lane, epi_pre &p, int ct = 0)
{
    const int j = ct * 16 + (lane & 15), g = lane >> 4;
    p.rj = 1.f; p.pos = 0; p.phys = 0;
    p.xo = make_float4(0.f, 0.f, 0.f, 0.f); p.gn = make_uint2(0u, 0u);
#pragma unroll
    for (int r = 0; r < 4; ++r) p.cs[r] = make_float2(1.f, 0.f);
    p.rows = a.st->gamma;
    if (EPI == EPI_RESID) {
        const int n = strip * 16 + 4 * g;
        if (j < p.rows) p.xo = *(const float4 *)(a.x + (size_t)j * a.d + n);
        p.gn = *(const uint2 *)(a.gain_next + n);
    }
    if (EPI == EPI_QKV) {
        // position and pages of row j: the cache's own, or in a batched step those of the row's sequence
        const int nseq = a.st->blk.n_seq;
        const int32_t *pt = a.page_table;
        int tag = 0;
        p.pos = a.st->len + j;
        if (nseq > 1 && j < p.rows) {
            const int sidx = a.st->rowseq[j];
            p.pos = a.st->rowpos[j]; pt = a.st->blk.seq[sidx].page_table; tag = (sidx + 1) << PV_SEQ_TAG_SHIFT;
        }
        if (j < p.rows) {
            if (strip >= a.q_strips) p.phys = pt[p.pos >> a.geom.page_shift] | tag;
            if (strip < a.q_strips + a.k_strips) {
                const int spH = a.geom.head_dim >> 4, tt = strip % spH, e = tt * 8 + 4 * (g >> 1);
#pragma unroll
                for (int r = 0; r < 4; ++r) p.cs[r] = a.rope[(size_t)j * (a.geom.head_dim >> 1) + e + r];
            }
        }
    }
}

// LDS hand-over of the prefetched inputs across the weight stream (they would otherwise occupy
// registers for the whole K loop): only the fields the epilogue kind reads travel.
template <int EPI>
__device__ inline void epi_park(epi_pre *slot, const epi_pre &p)
{
    slot->rows = p.rows;
    if (EPI == EPI_RESID) { slot->xo = p.xo; slot->gn = p.gn; }
    if (EPI == EPI_QKV) {
        slot->pos = p.pos; slot->phys = p.phys;
#pragma unroll
        for (int r = 0; r < 4; ++r) slot->cs[r] = p.cs[r];
    }
}

template <int EPI>
__device__ inline void epi_unpark(const epi_pre *slot, epi_pre &p)
{
    p.rj = 1.f; p.pos = 0; p.phys = 0;
    p.xo = make_float4(0.f, 0.f, 0.f, 0.f); p.gn = make_uint2(0u, 0u);
#pragma unroll
    for (int r = 0; r < 4; ++r) p.cs[r] = make_float2(1.f, 0.f);
    p.rows = slot->rows;
    if (EPI == EPI_RESID) { p.xo = slot->xo; p.gn = slot->gn; }
    if (EPI == EPI_QKV) {
        p.pos = slot->pos; p.phys = slot->phys;
#pragma unroll
        for (int r = 0; r < 4; ++r) p.cs[r] = slot->cs[r];
    }
}

// sum = the strip's accumulator (already summed over the K split)
template <int NB, int EPI>
__device__ inline void epi_apply(const gemm_args &a, int strip, int lane, f32x4 sum, const epi_pre &p, int ct = 0)
{
    constexpr bool NORM = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD);
    const int j = ct * 16 + (lane & 15), g = lane >> 4, rows = p.rows;
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = (NB == 1) ? sum[r] + __shfl_down(sum[r], 8, 64) : sum[r];   // hi + lo columns (lo_off == 4: the loads put the lo columns into 8..11 as well)
    const bool live = j < rows;          // NB == 1 implies rows <= 8, so live lanes hold the combined value
    if (NORM) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] *= p.rj;
    }

    if (EPI == EPI_QKV) {
        // the pages the row's keys and values go to: the cache's own, or (batched step) those of the row's sequence
        pv_kv_geom gm = a.geom;
        uint16_t *pool = a.pool;
        const int phys = p.phys & ((1 << PV_SEQ_TAG_SHIFT) - 1);
        if (p.phys >> PV_SEQ_TAG_SHIFT) {
            const pv_seq_ref &sq = a.st->blk.seq[(p.phys >> PV_SEQ_TAG_SHIFT) - 1];
            pool = (uint16_t *)sq.pool; gm.n_pages = sq.n_pages;
        }
        const int hd = gm.head_dim, half = hd >> 1, spH = hd >> 4;
        const int tok = p.pos & (gm.page_tokens - 1);
        if (strip < a.q_strips + a.k_strips) {
            const int h = strip / spH, tt = strip - h * spH, side = g & 1, e = tt * 8 + 4 * (g >> 1);
            float o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float partner = __shfl_xor(v[r], 16, 64);
                o[r] = side ? v[r] * p.cs[r].x + partner * p.cs[r].y : v[r] * p.cs[r].x - partner * p.cs[r].y;
            }
            if (live) {
                if (strip < a.q_strips) {
                    // queries leave as bf16 hi + lo pairs, the form attention feeds to the matrix cores
                    uint16_t qh[4], ql[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) { qh[r] = bf16_rne(o[r]); ql[r] = bf16_rne(o[r] - pv_bf16_to_f32(qh[r])); }
                    const size_t qo = ((size_t)j * a.n_q_heads + h) * hd + e + side * half;
                    *(uint2 *)(a.q_hi + qo) = make_uint2(qh[0] | ((uint32_t)qh[1] << 16), qh[2] | ((uint32_t)qh[3] << 16));
                    *(uint2 *)(a.q_lo + qo) = make_uint2(ql[0] | ((uint32_t)ql[1] << 16), ql[2] | ((uint32_t)ql[3] << 16));
                } else {
                    const int kvh = h - a.n_q_heads;
                    uint16_t *kp = pool + pv_kv_block(gm, a.layer, phys, kvh, 0) + pv_k_off(gm, tok, e + side * half);
                    *(uint2 *)kp = make_uint2(bf16_rne(o[0]) | ((uint32_t)bf16_rne(o[1]) << 16), bf16_rne(o[2]) | ((uint32_t)bf16_rne(o[3]) << 16));
                }
            }
        } else if (live) {
            const int sv = strip - a.q_strips - a.k_strips, kvh = sv / spH, e = (sv - kvh * spH) * 16 + 4 * g;
            uint16_t *vp = pool + pv_kv_block(gm, a.layer, phys, kvh, 1);
#pragma unroll
            for (int r = 0; r < 4; ++r) vp[pv_v_off(gm, tok, e + r)] = bf16_rne(v[r]);
        }
    } else if (EPI == EPI_RESID) {
        v[0] += p.xo.x; v[1] += p.xo.y; v[2] += p.xo.z; v[3] += p.xo.w;       // xo is zero on dead lanes
        emit_x<NB>(lane, rows, strip, a.d, v, p.gn, a.x, a.ssq_out, a.xop_out, ct, a.lo_off);
    } else if (EPI == EPI_SWIGLU) {
        float act[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float up = __shfl_xor(v[r], 16, 64);
            act[r] = v[r] / (1.0f + expf(-v[r])) * up;
        }
        if (live && !(g & 1)) store_operand4<NB>(a.xop_act, a.F, j, strip * 8 + 4 * (g >> 1), act, a.lo_off);
    } else {   // EPI_LMHEAD
        const int n = strip * 16 + 4 * g;
        if (live) *(float4 *)(a.logits + (size_t)j * a.vocab + n) = make_float4(v[0], v[1], v[2], v[3]);
        float bv = -INFINITY; int bi = 0x7fffffff;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float val = (v[r] == v[r]) ? v[r] : -INFINITY;
            if (val > bv || (val == bv && n + r < bi)) { bv = val; bi = n + r; }
        }
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            const float ov = __shfl_xor(bv, o, 64); const int oi = __shfl_xor(bi, o, 64);
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        // candidates are stored row-major ([16][vocab/16]) so that the reduction over strips reads contiguously
        if (lane < 16) { const size_t o = (size_t)j * (a.vocab >> 4) + strip; a.pmax_val[o] = bv; a.pmax_idx[o] = bi; }
    }
}
