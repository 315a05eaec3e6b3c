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
#include "pv_kernels_common.h"

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_LMHEAD = 3 };

struct mat_ws {                 // carved out of pv_ws::part
    uint16_t *xop_a, *xop_o, *xop_f, *xop_d;   // operands: QKV in (K=d), O in (K=qd), gate/up in (K=d), down in (K=F)
    float *ssq0, *ssq1;                         // [d/16][16] partial sums of x^2
    float *pmax_val; int32_t *pmax_idx;         // [vocab/16][16] per-strip arg-max candidates
};

static inline size_t xop_elems(int K) { return (size_t)2 * (K / 32) * 512; }   // hi and lo arrays

static size_t mat_ws_layout(const pv_model_config &f, float *base, mat_ws *w)
{
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
    return off;
}

size_t pv_mat_part_floats(const pv_model *m, int) { return mat_ws_layout(m->cfg, nullptr, nullptr); }

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

// ------------------------------------------------------------------------------------------
// Operand writers.  Element (row j, K-index k) of an activation lives at
//   arr[(k/32)*512 + (col + 16*((k%32)/8))*8 + k%8],  col = j (hi) / j+8 (lo) when NB == 1,
//   and col = j in the hi array / lo array when NB == 2.
// ------------------------------------------------------------------------------------------
__device__ inline uint16_t bf16_rne(float f) { return pv_f32_to_bf16(f); }

// four consecutive k (k0 % 4 == 0) of row j
template <int NB>
__device__ inline void store_operand4(uint16_t *xop, int K, int j, int k0, const float y[4])
{
    uint16_t hi[4], lo[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { hi[r] = bf16_rne(y[r]); lo[r] = bf16_rne(y[r] - pv_bf16_to_f32(hi[r])); }
    const size_t tile = (size_t)(k0 >> 5) * 512, in = (size_t)(((k0 & 31) >> 3) * 16) * 8 + (k0 & 7);
    const uint2 vh = make_uint2(hi[0] | ((uint32_t)hi[1] << 16), hi[2] | ((uint32_t)hi[3] << 16));
    const uint2 vl = make_uint2(lo[0] | ((uint32_t)lo[1] << 16), lo[2] | ((uint32_t)lo[3] << 16));
    if (NB == 1) {
        *(uint2 *)(xop + tile + in + (size_t)j * 8) = vh;
        *(uint2 *)(xop + tile + in + (size_t)(j + 8) * 8) = vl;
    } else {
        *(uint2 *)(xop + tile + in + (size_t)j * 8) = vh;
        *(uint2 *)(xop + (size_t)(K / 32) * 512 + tile + in + (size_t)j * 8) = vl;
    }
}

// Shared tail of everything that produces a new residual stream value: store x, the partial
// sum of squares of this 16-feature strip, and (gain * x) as the next GEMM's operand.
// Lane layout: j = lane % 16 (row), g = lane / 16, features n0 + 4g + r.
template <int NB>
__device__ inline void emit_x(int lane, int rows, int strip, int d, const float v[4], const uint16_t *gain,
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
        float y[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) y[r] = v[r] * pv_bf16_to_f32(gain[n + r]);
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
    emit_x<NB>(lane, rows, strip, d, v, gain, x, ssq, xop);
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

__device__ inline f32x4 mfma16(uint4 a, uint4 b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

template <int NB, int EPI>
__global__ void __launch_bounds__(512)
k_gemm(const gemm_args a)
{
    constexpr int U = 4;
    const int strip = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int KT = a.ktiles, per = (KT + 7) >> 3;
    const int kb = wave * per, ke = min(KT, kb + per);
    const uint4 *A = a.W + (size_t)strip * KT * 64 + lane;
    const uint4 *B = a.xop + lane;
    const uint4 *B2 = a.xop + (size_t)KT * 64 + lane;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};

    int t = kb;
    if (t + U <= ke) {
        uint4 a0[U], b0[U], c0[U], a1[U], b1[U], c1[U];
#define PV_LOAD(A_, B_, C_)                                                                   \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                       \
            A_[u] = A[(size_t)(t + u) * 64]; B_[u] = B[(size_t)(t + u) * 64];                 \
            if (NB == 2) C_[u] = B2[(size_t)(t + u) * 64];                                    \
        }                                                                                     \
        t += U;
#define PV_MMA(A_, B_, C_)                                                                    \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                       \
            acc = mfma16(A_[u], B_[u], acc);                                                  \
            if (NB == 2) acc = mfma16(A_[u], C_[u], acc);                                     \
        }
        PV_LOAD(a0, b0, c0)
        for (;;) {                       // two register buffers: loads of one overlap the MFMAs of the other
            if (t + U <= ke) { PV_LOAD(a1, b1, c1) PV_MMA(a0, b0, c0) } else { PV_MMA(a0, b0, c0) break; }
            if (t + U <= ke) { PV_LOAD(a0, b0, c0) PV_MMA(a1, b1, c1) } else { PV_MMA(a1, b1, c1) break; }
        }
#undef PV_LOAD
#undef PV_MMA
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

    const int j = lane & 15, g = lane >> 4, rows = a.st->gamma;
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = (NB == 1) ? sum[r] + __shfl_down(sum[r], 8, 64) : sum[r];
    const bool live = j < rows;          // NB == 1 implies rows <= 8, so live lanes hold the combined value

    if (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD) {
        float s = 0.f;
        for (int p = g; p < a.ssq_parts; p += 4) s += a.ssq[p * 16 + j];
        s += __shfl_xor(s, 16, 64);
        s += __shfl_xor(s, 32, 64);
        const float rj = 1.0f / sqrtf(s * a.inv_d + a.eps);
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] *= rj;
    }

    if (EPI == EPI_QKV) {
        const pv_kv_geom &gm = a.geom;
        const int hd = gm.head_dim, half = hd >> 1, spH = hd >> 4;
        const int pos = a.st->len + j;
        if (strip < a.q_strips + a.k_strips) {
            const int h = strip / spH, tt = strip - h * spH, side = g >> 1, e = tt * 8 + 4 * (g & 1);
            float o[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float partner = __shfl_xor(v[r], 32, 64);
                const float2 cs = live ? a.rope[(size_t)j * half + e + r] : make_float2(1.f, 0.f);
                o[r] = side ? v[r] * cs.x + partner * cs.y : v[r] * cs.x - partner * cs.y;
            }
            if (live) {
                if (strip < a.q_strips) {
                    *(float4 *)(a.q + ((size_t)j * a.n_q_heads + h) * hd + e + side * half) = make_float4(o[0], o[1], o[2], o[3]);
                } else {
                    const int kvh = h - a.n_q_heads;
                    const int phys = a.page_table[pos >> gm.page_shift], tok = pos & (gm.page_tokens - 1);
                    uint16_t *kp = a.pool + pv_kv_block(gm, a.layer, phys, kvh, 0) + (size_t)tok * hd + e + side * half;
                    *(uint2 *)kp = make_uint2(bf16_rne(o[0]) | ((uint32_t)bf16_rne(o[1]) << 16), bf16_rne(o[2]) | ((uint32_t)bf16_rne(o[3]) << 16));
                }
            }
        } else if (live) {
            const int sv = strip - a.q_strips - a.k_strips, kvh = sv / spH, e = (sv - kvh * spH) * 16 + 4 * g;
            const int phys = a.page_table[pos >> gm.page_shift], tok = pos & (gm.page_tokens - 1);
            uint16_t *vp = a.pool + pv_kv_block(gm, a.layer, phys, kvh, 1) + tok;
#pragma unroll
            for (int r = 0; r < 4; ++r) vp[(size_t)(e + r) * gm.page_tokens] = bf16_rne(v[r]);
        }
    } else if (EPI == EPI_RESID) {
        if (live) {
            const float4 xo = *(const float4 *)(a.x + (size_t)j * a.d + strip * 16 + 4 * g);
            v[0] += xo.x; v[1] += xo.y; v[2] += xo.z; v[3] += xo.w;
        }
        emit_x<NB>(lane, rows, strip, a.d, v, a.gain_next, a.x, a.ssq_out, a.xop_out);
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
    mat_ws_layout(f, c->ws.part, &mw);
    const char *Wb = m->d_weights;
    auto gainp = [&](int kind, int l) { return (const uint16_t *)(Wb + pv_tref(m, kind, l).off); };

    k_mat_begin<NB><<<d / 16, 64, 0, s>>>(c->ws.state, (const uint16_t *)(Wb + m->global[PV_T_EMBED].off), gainp(PV_T_ATTN_NORM, 0),
                                           (const double *)(Wb + m->inv_freq_off), c->ws.x, mw.ssq0, mw.xop_a, c->ws.rope, d, hd / 2);
    PV_HIP(hipGetLastError());

    gemm_args g = {};
    g.st = c->ws.state; g.inv_d = 1.0f / (float)d; g.eps = (float)f.rms_eps; g.ssq_parts = d / 16;
    g.q = c->ws.q; g.pool = (uint16_t *)c->d_pool; g.page_table = c->ws.page_table; g.rope = c->ws.rope; g.geom = pv_geom(c);
    g.n_q_heads = f.n_q_heads; g.q_strips = qd / 16; g.k_strips = kvd / 16;
    g.x = c->ws.x; g.d = d; g.xop_act = mw.xop_d; g.F = F;
    g.logits = c->ws.logits; g.pmax_val = mw.pmax_val; g.pmax_idx = mw.pmax_idx; g.vocab = f.vocab;

    for (int l = 0; l < f.n_layers; ++l) {
        // fused QKV projection: RMSNorm scale, rotary embedding, KV append
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WQ, l).off); g.xop = (const uint4 *)mw.xop_a; g.ktiles = d / 32;
        g.ssq = mw.ssq0; g.layer = l;
        k_gemm<NB, EPI_QKV><<<(qd + 2 * kvd) / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        // attention (vector kernel for now) -> operand of the output projection
        int rc = pv_vec_attention_bf16(c, l, rows, s);
        if (rc != PV_OK) return rc;
        k_to_operand<NB><<<(rows * (qd / 4) + 255) / 256, 256, 0, s>>>(c->ws.state, c->ws.attn, mw.xop_o, qd);
        PV_HIP(hipGetLastError());
        // output projection + residual; emits the FFN operand and sum of squares
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WO, l).off); g.xop = (const uint4 *)mw.xop_o; g.ktiles = qd / 32;
        g.gain_next = gainp(PV_T_FFN_NORM, l); g.ssq_out = mw.ssq1; g.xop_out = mw.xop_f;
        k_gemm<NB, EPI_RESID><<<d / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        // gate/up projection + SwiGLU
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WG, l).off); g.xop = (const uint4 *)mw.xop_f; g.ktiles = d / 32;
        g.ssq = mw.ssq1;
        k_gemm<NB, EPI_SWIGLU><<<F / 8, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
        // down projection + residual; emits the next layer's (or the head's) operand
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WD, l).off); g.xop = (const uint4 *)mw.xop_d; g.ktiles = F / 32;
        g.gain_next = (l + 1 < f.n_layers) ? gainp(PV_T_ATTN_NORM, l + 1) : (const uint16_t *)(Wb + m->global[PV_T_FINAL_NORM].off);
        g.ssq_out = mw.ssq0; g.xop_out = mw.xop_a;
        k_gemm<NB, EPI_RESID><<<d / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
    }
    const bool head = c->io->hdr[3] != PV_MODE_PREFILL_MID;
    if (head) {
        g.W = (const uint4 *)(Wb + m->global[PV_T_LM_HEAD].off); g.xop = (const uint4 *)mw.xop_a; g.ktiles = d / 32; g.ssq = mw.ssq0;
        k_gemm<NB, EPI_LMHEAD><<<f.vocab / 16, 512, 0, s>>>(g);
        PV_HIP(hipGetLastError());
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
