// Matrix-core kernel family for bf16 models.
//
// Skinny GEMMs y[rows<=16][N] = x[rows][K] W^T stream W once from HBM.  W is stored pre-tiled
// in MFMA operand order: strips of 16 output features, each strip a run of K/32 tiles of
// 16x32 bf16 (1 KiB), a tile laid out [lane 0..63][8 bf16] so that one 16-byte load per lane
// is exactly the A operand of v_mfma_f32_16x16x32_bf16.  A workgroup owns one strip: its 8
// wavefronts split K, accumulate in fp32, and are summed in wave order through LDS, so the
// owner sees complete outputs and the whole epilogue (RMSNorm scale, rotary embedding + KV
// append, SwiGLU, residual add, vocabulary arg-max) is fused into the GEMM.
//
// Activations enter as the B operand.  To keep fp32-grade accuracy with bf16 matrix cores an
// activation a is carried as two bf16 numbers hi = bf16(a), lo = bf16(a - hi) (16 mantissa
// bits).  For rows <= 8 the 16 operand columns hold hi of row j in column j and lo in column
// j+8, so one MFMA does both and the epilogue adds the two column halves; for 9..16 rows hi
// and lo are separate operands and two MFMAs accumulate into the same registers.
//
// RMSNorm is folded in: the producer of x writes (gain * x) as the next operand plus per-strip
// partial sums of x^2; the consumer multiplies its outputs by rsqrt(mean + eps), which
// commutes with the contraction.  Rows of W_q/W_k are permuted inside each head so that the two
// members of a rotary pair sit in the same strip 8 rows apart (lanes l and l^32 of the
// accumulator); gate and up rows are interleaved the same way for SwiGLU.
#include "pv_matrix_common.h"


enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

struct mat_ws {                 // carved out of pv_ws::part
    uint16_t *xop_a, *xop_o, *xop_f, *xop_d;   // operands: QKV in (K=d), O in (K=qd), gate/up in (K=d), down in (K=F)
    float *ssq0, *ssq1;                         // [d/16][16] partial sums of x^2
    float *pmax_val; int32_t *pmax_idx;         // [vocab/16][16] per-strip arg-max candidates
    float *attn_part;                           // attention chunk partials
};

static inline size_t xop_elems(int K) { return (size_t)2 * (K / 32) * 512; }   // hi and lo arrays

static size_t mat_ws_layout(const pv_model *m, int rows_cap, int max_tokens, float *base, mat_ws *w)
{
    const pv_model_config &f = m->cfg;
    const int qd = f.n_q_heads * f.head_dim;
    size_t off = 0;   // in floats, every piece a multiple of 64 floats (256 B)
    auto take = [&](size_t floats) { size_t o = off; off += (floats + 63) / 64 * 64; return base ? base + o : (float *)nullptr; };
    float *p;
    p = take(xop_elems(f.d_model) / 2); if (w) w->xop_a = (uint16_t *)p;
    p = take(xop_elems(qd) / 2); if (w) w->xop_o = (uint16_t *)p;
    p = take(xop_elems(f.d_model) / 2); if (w) w->xop_f = (uint16_t *)p;
    p = take(xop_elems(f.ffn_dim) / 2); if (w) w->xop_d = (uint16_t *)p;
    p = take((size_t)f.d_model); if (w) w->ssq0 = p;
    p = take((size_t)f.d_model); if (w) w->ssq1 = p;
    p = take((size_t)f.vocab); if (w) w->pmax_val = p;
    p = take((size_t)f.vocab); if (w) w->pmax_idx = (int32_t *)p;
    p = take(pv_attn_part_floats(m, rows_cap, max_tokens)); if (w) w->attn_part = p;
    return off;
}

size_t pv_mat_part_floats(const pv_model *m, int rows_cap, int max_tokens) { return mat_ws_layout(m, rows_cap, max_tokens, nullptr, nullptr); }

// ------------------------------------------------------------------------------------------
// Weight repack: rows [row_begin, row_begin+row_count) of one tensor, row-major in staging,
// into the tiled region.  One thread moves 8 consecutive K elements (16 bytes).
// ------------------------------------------------------------------------------------------
enum { PERM_NONE = 0, PERM_ROPE = 1, PERM_GATEUP = 2 };

__global__ void k_repack(const uint4 *src, uint4 *dst, int64_t row_begin, int64_t row_count, int K,
                         int perm, int head_dim, int strip_mul, int strip_add)
{
    const int kg = K / 8;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= row_count * kg) return;
    const int64_t n = row_begin + idx / kg;
    const int kb = (int)(idx % kg);                 // group of 8 along K
    int64_t strip; int i;
    if (perm == PERM_ROPE) {
        const int half = head_dim / 2, e = (int)(n % head_dim);
        const int64_t h = n / head_dim;
        const int side = e >= half, p = e - side * half;
        strip = h * (head_dim / 16) + p / 8; i = (p & 7) + 8 * side;
    } else if (perm == PERM_GATEUP) {
        strip = n / 8; i = (int)(n & 7) + 8 * strip_add;         // strip_add: 0 = gate, 1 = up
    } else {
        strip = (n / 16) * strip_mul + strip_add; i = (int)(n & 15);
    }
    const int kt = kb / 4, lane = i + 16 * (kb & 3);
    dst[((size_t)strip * (K / 32) + kt) * 64 + lane] = src[idx];
}

int pv_mat_repack(const pv_model *m, const pv_tensor_ref &t, int kind, int64_t row_begin, int64_t row_count, hipStream_t s)
{
    int perm = PERM_NONE, mul = 1, add = 0;
    if (kind == PV_T_WQ || kind == PV_T_WK) perm = PERM_ROPE;
    else if (kind == PV_T_WG || kind == PV_T_WU) { perm = PERM_GATEUP; add = t.strip_add; }
    const int64_t n = row_count * (t.cols / 8);
    k_repack<<<(unsigned)((n + 255) / 256), 256, 0, s>>>((const uint4 *)m->d_staging, (uint4 *)(m->d_weights + t.off),
                                                         row_begin, row_count, (int)t.cols, perm, m->cfg.head_dim, mul, add);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

// Shared tail of everything that produces a new residual stream value: store x, the partial
// sum of squares of this 16-feature strip, and (gain * x) as the next GEMM's operand.
// Lane layout: j = lane % 16 (row), g = lane / 16, features n0 + 4g + r.
template <int NB>
__device__ inline void emit_x(int lane, int rows, int strip, int d, const float v[4], uint2 gain4,
                              float *x, float *ssq, uint16_t *xop)
{
    const int j = lane & 15, g = lane >> 4, n = strip * 16 + 4 * g;
    const bool live = j < rows;
    if (live) *(float4 *)(x + (size_t)j * d + n) = make_float4(v[0], v[1], v[2], v[3]);
    float ss = live ? (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]) : 0.f;
    ss += __shfl_xor(ss, 16, 64);
    ss += __shfl_xor(ss, 32, 64);
    if (lane < 16) ssq[strip * 16 + j] = ss;
    if (live) {
        const float y[4] = {v[0] * pv_bf16_to_f32((uint16_t)(gain4.x & 0xffffu)), v[1] * pv_bf16_to_f32((uint16_t)(gain4.x >> 16)),
                            v[2] * pv_bf16_to_f32((uint16_t)(gain4.y & 0xffffu)), v[3] * pv_bf16_to_f32((uint16_t)(gain4.y >> 16))};
        store_operand4<NB>(xop, d, j, n, y);
    }
}

// Block set-up on the matrix path: embedding rows -> x, first operand, first sum of squares;
// rotary table for positions len .. len+rows-1.
template <int NB>
__global__ void __launch_bounds__(64)
k_mat_begin(const pv_dev_state *st, const uint16_t *embed, const uint16_t *gain, const double *inv_freq,
            float *x, float *ssq, uint16_t *xop, float2 *rope, int d, int half)
{
    const int lane = threadIdx.x, j = lane & 15, g = lane >> 4, rows = st->gamma, strip = blockIdx.x;
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (j < rows) {
        const uint16_t *e = embed + (size_t)st->draft[j] * d + strip * 16 + 4 * g;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = pv_bf16_to_f32(e[r]);
    }
    emit_x<NB>(lane, rows, strip, d, v, *(const uint2 *)(gain + strip * 16 + 4 * g), x, ssq, xop);
    for (int idx = blockIdx.x * 64 + lane; idx < rows * half; idx += gridDim.x * 64) {
        const int jj = idx / half, i = idx - jj * half;
        double sn, cs;
        sincos((double)(st->len + jj) * inv_freq[i], &sn, &cs);
        rope[idx] = make_float2((float)cs, (float)sn);
    }
}

// fp32 [rows][K] -> operand (no gain); used for the attention output
template <int NB>
__global__ void k_to_operand(const pv_dev_state *st, const float *src, uint16_t *xop, int K)
{
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;       // (row, group of 4)
    const int per_row = K / 4, j = idx / per_row, k0 = (idx - j * per_row) * 4;
    if (j >= st->gamma) return;
    const float4 a = *(const float4 *)(src + (size_t)j * K + k0);
    const float y[4] = {a.x, a.y, a.z, a.w};
    store_operand4<NB>(xop, K, j, k0, y);
}

// ------------------------------------------------------------------------------------------
// The streaming GEMM.
// ------------------------------------------------------------------------------------------
struct gemm_args {
    const uint4 *W;             // tiled region, strip-major
    const uint4 *xop;           // operand (hi [+ lo array behind it when NB == 2])
    int ktiles;                 // K / 32
    const pv_dev_state *st;
    // RMSNorm scale of the input rows (QKV, SWIGLU, LMHEAD)
    const float *ssq; int ssq_parts; float inv_d, eps;
    // QKV
    float *q; uint16_t *pool; const int32_t *page_table; const float2 *rope; pv_kv_geom geom;
    int layer, n_q_heads, q_strips, k_strips;
    // RESID
    float *x; const uint16_t *gain_next; float *ssq_out; uint16_t *xop_out; int d;
    // SWIGLU
    uint16_t *xop_act; int F;
    // LMHEAD
    float *logits; float *pmax_val; int32_t *pmax_idx; int vocab;
};


// rsqrt(mean(x_j^2) + eps) for row j = lane % 16 from the [parts][16] partial sums, summed in a
// fixed order.  All loads are independent (a serial chain of L2 round trips would cost far more
// than the weight stream it sits beside): lane l reads float4 number l, l+64, ... so it always
// sees rows 4*(l%4)..+3; lanes with equal l%4 are then combined and the result redistributed.
__device__ inline float row_rscale(const float *ssq, int parts, float inv_d, float eps, int lane)
{
    const float4 *q = (const float4 *)ssq;
    const int n4 = parts * 4;
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i0 = lane; i0 < n4; i0 += 64 * 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { const int i = i0 + u * 64; v[u] = i < n4 ? q[i] : make_float4(0.f, 0.f, 0.f, 0.f); }
#pragma unroll
        for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
#pragma unroll
    for (int o = 4; o <= 32; o <<= 1) {
        s.x += __shfl_xor(s.x, o, 64); s.y += __shfl_xor(s.y, o, 64); s.z += __shfl_xor(s.z, o, 64); s.w += __shfl_xor(s.w, o, 64);
    }
    const int j = lane & 15, src = j >> 2;
    const float t0 = __shfl(s.x, src, 64), t1 = __shfl(s.y, src, 64), t2 = __shfl(s.z, src, 64), t3 = __shfl(s.w, src, 64);
    const float tot = (j & 3) == 0 ? t0 : (j & 3) == 1 ? t1 : (j & 3) == 2 ? t2 : t3;
    return 1.0f / sqrtf(tot * inv_d + eps);
}

template <int NB, int EPI>
__global__ void __launch_bounds__(512)
k_gemm(const gemm_args a)
{
    constexpr int U = 4;
    constexpr bool NORM = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD);
    const int strip = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int KT = a.ktiles, per = (KT + 7) >> 3;
    const int kb = wave * per, ke = min(KT, kb + per);
    const uint4 *A = a.W + (size_t)strip * KT * 64 + lane;
    const uint4 *B = a.xop + lane;
    const uint4 *B2 = a.xop + (size_t)KT * 64 + lane;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};

    // The owner wave fetches what its epilogue needs before streaming, so that after the
    // reduction only arithmetic and stores remain: rsqrt(mean(x^2)+eps) of its row.
    float rj = 1.f;
    int rows = 0, pos = 0, phys = 0;
    float4 xo = make_float4(0.f, 0.f, 0.f, 0.f);
    uint2 gn = make_uint2(0u, 0u);
    float2 cs[4] = {make_float2(1.f, 0.f), make_float2(1.f, 0.f), make_float2(1.f, 0.f), make_float2(1.f, 0.f)};
    if (wave == 0) {
        const int j = lane & 15, g = lane >> 4;
        rows = a.st->gamma;
        if (NORM) rj = row_rscale(a.ssq, a.ssq_parts, a.inv_d, a.eps, lane);
        if (EPI == EPI_RESID) {
            const int n = strip * 16 + 4 * g;
            if (j < rows) xo = *(const float4 *)(a.x + (size_t)j * a.d + n);
            gn = *(const uint2 *)(a.gain_next + n);
        }
        if (EPI == EPI_QKV) {
            pos = a.st->len + j;
            if (j < rows) {
                if (strip >= a.q_strips) phys = a.page_table[pos >> a.geom.page_shift];
                if (strip < a.q_strips + a.k_strips) {
                    const int spH = a.geom.head_dim >> 4, tt = strip % spH, e = tt * 8 + 4 * (g & 1);
#pragma unroll
                    for (int r = 0; r < 4; ++r) cs[r] = a.rope[(size_t)j * (a.geom.head_dim >> 1) + e + r];
                }
            }
        }
    }

    // Few registers on purpose: latency is hidden by many resident workgroups per CU.
    int t = kb;
    for (; t + U <= ke; t += U) {
        uint4 ra[U], rb[U], rc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            ra[u] = A[(size_t)(t + u) * 64]; rb[u] = B[(size_t)(t + u) * 64];
            if (NB == 2) rc[u] = B2[(size_t)(t + u) * 64];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc = mfma16(ra[u], rb[u], acc);
            if (NB == 2) acc = mfma16(ra[u], rc[u], acc);
        }
    }
    for (; t < ke; ++t) {
        acc = mfma16(A[(size_t)t * 64], B[(size_t)t * 64], acc);
        if (NB == 2) acc = mfma16(A[(size_t)t * 64], B2[(size_t)t * 64], acc);
    }

    // sum the 8 K-slices in wave order
    __shared__ f32x4 red[8][64];
    red[wave][lane] = acc;
    __syncthreads();
    if (wave != 0) return;
    f32x4 sum = red[0][lane];
#pragma unroll
    for (int w = 1; w < 8; ++w) { const f32x4 p = red[w][lane]; sum[0] += p[0]; sum[1] += p[1]; sum[2] += p[2]; sum[3] += p[3]; }

    const int j = lane & 15, g = lane >> 4;
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = (NB == 1) ? sum[r] + __shfl_down(sum[r], 8, 64) : sum[r];
    const bool live = j < rows;          // NB == 1 implies rows <= 8, so live lanes hold the combined value

    if (NORM) {
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] *= rj;
    }

    if (EPI == EPI_QKV) {
        const pv_kv_geom &gm = a.geom;
        const int hd = gm.head_dim, half = hd >> 1, spH = hd >> 4;
        if (strip < a.q_strips + a.k_strips) {
            const int h = strip / spH, tt = strip - h * spH, side = g >> 1, e = tt * 8 + 4 * (g & 1);
            float o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float partner = __shfl_xor(v[r], 32, 64);
                o[r] = side ? v[r] * cs[r].x + partner * cs[r].y : v[r] * cs[r].x - partner * cs[r].y;
            }
            if (live) {
                if (strip < a.q_strips) {
                    *(float4 *)(a.q + ((size_t)j * a.n_q_heads + h) * hd + e + side * half) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
                    const int kvh = h - a.n_q_heads;
                    const int tok = pos & (gm.page_tokens - 1);
                    uint16_t *kp = a.pool + pv_kv_block(gm, a.layer, phys, kvh, 0) + pv_k_off(gm, tok, e + side * half);
                    *(uint2 *)kp = make_uint2(bf16_rne(o[0]) | ((uint32_t)bf16_rne(o[1]) << 16), bf16_rne(o[2]) | ((uint32_t)bf16_rne(o[3]) << 16));
                }
            }
        } else if (live) {
            const int sv = strip - a.q_strips - a.k_strips, kvh = sv / spH, e = (sv - kvh * spH) * 16 + 4 * g;
            const int tok = pos & (gm.page_tokens - 1);
            uint16_t *vp = a.pool + pv_kv_block(gm, a.layer, phys, kvh, 1);
#pragma unroll
            for (int r = 0; r < 4; ++r) vp[pv_v_off(gm, tok, e + r)] = bf16_rne(v[r]);
        }
    } else if (EPI == EPI_RESID) {
        v[0] += xo.x; v[1] += xo.y; v[2] += xo.z; v[3] += xo.w;       // xo is zero on dead lanes
        emit_x<NB>(lane, rows, strip, a.d, v, gn, a.x, a.ssq_out, a.xop_out);
    } else if (EPI == EPI_SWIGLU) {
        float act[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float up = __shfl_xor(v[r], 32, 64);
            act[r] = v[r] / (1.0f + expf(-v[r])) * up;
        }
        if (live && g < 2) store_operand4<NB>(a.xop_act, a.F, j, strip * 8 + 4 * g, act);
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
        if (lane < 16) { a.pmax_val[strip * 16 + j] = bv; a.pmax_idx[strip * 16 + j] = bi; }
    }
}

// arg-max over the per-strip candidates of one row
__global__ void __launch_bounds__(256)
k_argmax_parts(pv_dev_state *st, const float *pv, const int32_t *pi, int strips)
{
    const int j = blockIdx.x;
    if (j >= st->gamma) return;
    float bv = -INFINITY; int bi = 0x7fffffff;
    for (int s = threadIdx.x; s < strips; s += 256) {
        const float v = pv[s * 16 + j]; const int i = pi[s * 16 + j];
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
    __shared__ float sv[256];
    __shared__ int si[256];
    sv[threadIdx.x] = bv; si[threadIdx.x] = bi;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            const float ov = sv[threadIdx.x + s]; const int oi = si[threadIdx.x + s];
            if (ov > sv[threadIdx.x] || (ov == sv[threadIdx.x] && oi < si[threadIdx.x])) { sv[threadIdx.x] = ov; si[threadIdx.x] = oi; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) st->pred[j] = si[0];
}

// ------------------------------- host side ----------------------------------------

int pv_vec_attention_bf16(pv_cache *c, int layer, int rows, hipStream_t s);   // pv_kernels_vector.hip

template <int NB>
static int run_block(pv_cache *c, hipStream_t s)
{
    const pv_model *m = c->m;
    const pv_model_config &f = m->cfg;
    const int rows = c->last_rows, d = f.d_model, hd = f.head_dim, qd = f.n_q_heads * hd, kvd = f.n_kv_heads * hd, F = f.ffn_dim;
    mat_ws mw;
    mat_ws_layout(m, c->rows_cap, c->n_pages * f.page_tokens, c->ws.part, &mw);
    const char *Wb = m->d_weights;
    auto gainp = [&](int kind, int l) { return (const uint16_t *)(Wb + pv_tref(m, kind, l).off); };

    k_mat_begin<NB><<<d / 16, 64, 0, s>>>(c->ws.state, (const uint16_t *)(Wb + m->global[PV_T_EMBED].off), gainp(PV_T_ATTN_NORM, 0),
                                           (const double *)(Wb + m->inv_freq_off), c->ws.x, mw.ssq0, mw.xop_a, c->ws.rope, d, hd / 2);
    PV_HIP(hipGetLastError());

    gemm_args g = {};
    int prc;
    g.st = c->ws.state; g.inv_d = 1.0f / (float)d; g.eps = (float)f.rms_eps; g.ssq_parts = d / 16;
    g.q = c->ws.q; g.pool = (uint16_t *)c->d_pool; g.page_table = c->ws.page_table; g.rope = c->ws.rope; g.geom = pv_geom(c);
    g.n_q_heads = f.n_q_heads; g.q_strips = qd / 16; g.k_strips = kvd / 16;
    g.x = c->ws.x; g.d = d; g.xop_act = mw.xop_d; g.F = F;
    g.logits = c->ws.logits; g.pmax_val = mw.pmax_val; g.pmax_idx = mw.pmax_idx; g.vocab = f.vocab;

    for (int l = 0; l < f.n_layers; ++l) {
        // fused QKV projection: RMSNorm scale, rotary embedding, KV append
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WQ, l).off); g.xop = (const uint4 *)mw.xop_a; g.ktiles = d / 32;
        g.ssq = mw.ssq0; g.layer = l;
        if ((prc = pv_prof_mark(c, PV_PROF_QKV, l, 0, s)) != PV_OK) return prc;
        k_gemm<NB, EPI_QKV><<<(qd + 2 * kvd) / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        if ((prc = pv_prof_mark(c, PV_PROF_QKV, l, 1, s)) != PV_OK) return prc;
        // attention over the paged cache -> operand of the output projection
        if ((prc = pv_prof_mark(c, PV_PROF_ATTENTION, l, 0, s)) != PV_OK) return prc;
        int rc = pv_mat_attention(c, l, rows, mw.attn_part, mw.xop_o, s);
        if (rc != PV_OK) return rc;
        if ((prc = pv_prof_mark(c, PV_PROF_ATTENTION, l, 1, s)) != PV_OK) return prc;
        // output projection + residual; emits the FFN operand and sum of squares
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WO, l).off); g.xop = (const uint4 *)mw.xop_o; g.ktiles = qd / 32;
        g.gain_next = gainp(PV_T_FFN_NORM, l); g.ssq_out = mw.ssq1; g.xop_out = mw.xop_f;
        if ((prc = pv_prof_mark(c, PV_PROF_OPROJ, l, 0, s)) != PV_OK) return prc;
        k_gemm<NB, EPI_RESID><<<d / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        if ((prc = pv_prof_mark(c, PV_PROF_OPROJ, l, 1, s)) != PV_OK) return prc;
        // gate/up projection + SwiGLU
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WG, l).off); g.xop = (const uint4 *)mw.xop_f; g.ktiles = d / 32;
        g.ssq = mw.ssq1;
        if ((prc = pv_prof_mark(c, PV_PROF_GATEUP, l, 0, s)) != PV_OK) return prc;
        k_gemm<NB, EPI_SWIGLU><<<F / 8, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        if ((prc = pv_prof_mark(c, PV_PROF_GATEUP, l, 1, s)) != PV_OK) return prc;
        // down projection + residual; emits the next layer's (or the head's) operand
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WD, l).off); g.xop = (const uint4 *)mw.xop_d; g.ktiles = F / 32;
        g.gain_next = (l + 1 < f.n_layers) ? gainp(PV_T_ATTN_NORM, l + 1) : (const uint16_t *)(Wb + m->global[PV_T_FINAL_NORM].off);
        g.ssq_out = mw.ssq0; g.xop_out = mw.xop_a;
        if ((prc = pv_prof_mark(c, PV_PROF_DOWN, l, 0, s)) != PV_OK) return prc;
        k_gemm<NB, EPI_RESID><<<d / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        if ((prc = pv_prof_mark(c, PV_PROF_DOWN, l, 1, s)) != PV_OK) return prc;
    }
    const bool head = c->io->hdr[3] != PV_MODE_PREFILL_MID;
    if (head) {
        g.W = (const uint4 *)(Wb + m->global[PV_T_LM_HEAD].off); g.xop = (const uint4 *)mw.xop_a; g.ktiles = d / 32; g.ssq = mw.ssq0;
        if ((prc = pv_prof_mark(c, PV_PROF_LMHEAD, 0, 0, s)) != PV_OK) return prc;
        k_gemm<NB, EPI_LMHEAD><<<f.vocab / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        if ((prc = pv_prof_mark(c, PV_PROF_LMHEAD, 0, 1, s)) != PV_OK) return prc;
        k_argmax_parts<<<rows, 256, 0, s>>>(c->ws.state, mw.pmax_val, mw.pmax_idx, f.vocab / 16);
        PV_HIP(hipGetLastError());
    }
    return pv_k_argmax_accept(c, rows, false, s);
}

int pv_mat_run_block(pv_cache *c, hipStream_t s)
{
    if (c->last_rows > 16) { pv_set_error("matrix path handles at most 16 rows per block"); return PV_ERANGE; }
    return c->last_rows <= 8 ? run_block<1>(c, s) : run_block<2>(c, s);
}
