// Vector-ALU kernel family: row-major weights of any storage type, fp32 arithmetic.
// This is the path of fp32 models (the tiny parity configuration) and a second, structurally
// different GPU implementation that the matrix-core path can be cross-checked against.
// Every reduction has a fixed order, so repeated runs give identical bits.
#include "pv_kernels_common.h"

// ---- block-wide reductions through LDS, fixed tree order ----
template <int NT>
__device__ inline float block_sum(float v, float *red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = NT / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

template <int NT>
__device__ inline float block_max(float v, float *red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = NT / 2; s > 0; s >>= 1) {
        if (threadIdx.x < s) red[threadIdx.x] = fmaxf(red[threadIdx.x], red[threadIdx.x + s]);
        __syncthreads();
    }
    const float r = red[0];
    __syncthreads();
    return r;
}

// h[j,:] = x[j,:] * rsqrt(mean(x[j,:]^2) + eps) * g
template <typename ST>
__global__ void __launch_bounds__(256)
k_rmsnorm(const float *x, const ST *g, float *h, int d, float eps)
{
    __shared__ float red[256];
    const float *xr = x + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int i = threadIdx.x; i < d; i += 256) ss += xr[i] * xr[i];
    ss = block_sum<256>(ss, red);
    const float r = 1.0f / sqrtf(ss / (float)d + eps);
    for (int i = threadIdx.x; i < d; i += 256) h[(size_t)blockIdx.x * d + i] = xr[i] * r * pv_ld(g, i);
}

// y[g][n] = (res ? res[g][n] : 0) + sum_k x[g][k] * W[n][k]   for g < G rows; one wavefront per n.
// K must be a multiple of 4.  Rows >= `rows` are computed from padding and not stored.
template <typename ST, int G>
__global__ void __launch_bounds__(256)
k_linear(const ST *W, const float *x, const float *res, float *y, int N, int K, int rows)
{
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const ST *w = W + (size_t)n * K;
    float acc[G];
#pragma unroll
    for (int g = 0; g < G; ++g) acc[g] = 0.f;
    for (int k = lane * 4; k < K; k += 256) {
        const float w0 = pv_ld(w, k), w1 = pv_ld(w, k + 1), w2 = pv_ld(w, k + 2), w3 = pv_ld(w, k + 3);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float4 xv = *(const float4 *)(x + (size_t)g * K + k);
            acc[g] += xv.x * w0 + xv.y * w1 + xv.z * w2 + xv.w * w3;
        }
    }
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float a = acc[g];
        for (int o = 32; o > 0; o >>= 1) a += __shfl_xor(a, o, 64);
        if (lane == 0 && g < rows) y[(size_t)g * N + n] = (res ? res[(size_t)g * N + n] : 0.f) + a;
    }
}

// act = silu(gate) * up
__global__ void k_swiglu(const float *gate, const float *up, float *act, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { const float z = gate[i]; act[i] = z / (1.0f + expf(-z)) * up[i]; }
}

// Causal attention for one (query head, row): keys 0 .. len+j, streaming softmax over chunks
// of 1024 keys.  K/V come from the paged pool.
template <typename ST>
__global__ void __launch_bounds__(256)
k_attention(const pv_dev_state *st, const int32_t *page_table, const float *q, const ST *pool, float *out,
            pv_kv_geom g, int layer, int n_q_heads)
{
    const int j = blockIdx.y, a = blockIdx.x;
    if (j >= st->gamma) return;
    const int hd = g.head_dim, kvh = a / (n_q_heads / g.n_kv_heads);
    const int nkeys = st->len + j + 1;
    __shared__ float qs[256], sc[1024], red[256];
    if ((int)threadIdx.x < hd) qs[threadIdx.x] = q[((size_t)j * n_q_heads + a) * hd + threadIdx.x];
    __syncthreads();
    const float scale = 1.0f / sqrtf((float)hd);
    float m = -INFINITY, l = 0.f, o = 0.f;
    for (int c0 = 0; c0 < nkeys; c0 += 1024) {
        const int cn = min(1024, nkeys - c0);
        float lm = -INFINITY;
        for (int t = threadIdx.x; t < cn; t += 256) {
            const int p = c0 + t;
            const ST *kb = pool + pv_kv_block(g, layer, page_table[p >> g.page_shift], kvh, 0);
            const int tk = p & (g.page_tokens - 1);
            float s = 0.f;
            for (int e = 0; e < hd; ++e) s += qs[e] * pv_ld(kb, pv_k_off(g, tk, e));
            s *= scale;
            sc[t] = s;
            lm = fmaxf(lm, s);
        }
        const float m_new = fmaxf(m, block_max<256>(lm, red));
        float ls = 0.f;
        for (int t = threadIdx.x; t < cn; t += 256) { const float w = expf(sc[t] - m_new); sc[t] = w; ls += w; }
        const float cs = block_sum<256>(ls, red);          // also orders the sc[] writes before the reads below
        const float resc = expf(m - m_new);
        l = l * resc + cs;
        if ((int)threadIdx.x < hd) {
            float acc = 0.f;
            for (int t = 0; t < cn; ++t) {
                const int p = c0 + t;
                const ST *vb = pool + pv_kv_block(g, layer, page_table[p >> g.page_shift], kvh, 1);
                acc += sc[t] * pv_ld(vb, pv_v_off(g, p & (g.page_tokens - 1), threadIdx.x));
            }
            o = o * resc + acc;
        }
        m = m_new;
        __syncthreads();
    }
    if ((int)threadIdx.x < hd) out[((size_t)j * n_q_heads + a) * hd + threadIdx.x] = o / l;
}

// ------------------------------- host side ----------------------------------------

template <typename ST>
static int launch_linear(const pv_model *m, const pv_tensor_ref &t, const float *x, const float *res, float *y,
                         int rows, hipStream_t s)
{
    const ST *W = (const ST *)(m->d_weights + t.off);
    const int N = (int)t.rows, K = (int)t.cols;
    const unsigned grid = (unsigned)((N + 3) / 4);
    for (int r0 = 0; r0 < rows; r0 += 16) {
        const int r = rows - r0 < 16 ? rows - r0 : 16;
        const float *xr = x + (size_t)r0 * K, *rr = res ? res + (size_t)r0 * N : nullptr;
        float *yr = y + (size_t)r0 * N;
        if (r <= 1) k_linear<ST, 1><<<grid, 256, 0, s>>>(W, xr, rr, yr, N, K, r);
        else if (r <= 4) k_linear<ST, 4><<<grid, 256, 0, s>>>(W, xr, rr, yr, N, K, r);
        else if (r <= 8) k_linear<ST, 8><<<grid, 256, 0, s>>>(W, xr, rr, yr, N, K, r);
        else k_linear<ST, 16><<<grid, 256, 0, s>>>(W, xr, rr, yr, N, K, r);
        PV_HIP(hipGetLastError());
    }
    return PV_OK;
}

template <typename ST>
static int run_block(pv_cache *c, hipStream_t s)
{
    const pv_model *m = c->m;
    const pv_model_config &f = m->cfg;
    const int rows = c->last_rows, rows_pad = (rows + PV_ROW_PAD - 1) / PV_ROW_PAD * PV_ROW_PAD;
    const int d = f.d_model, qd = f.n_q_heads * f.head_dim, F = f.ffn_dim;
    const pv_kv_geom g = pv_geom(c);
    pv_ws &w = c->ws;
    int rc;
    if ((rc = pv_k_begin(c, rows_pad, s)) != PV_OK) return rc;
    for (int l = 0; l < f.n_layers; ++l) {
        k_rmsnorm<ST><<<rows, 256, 0, s>>>(w.x, (const ST *)(m->d_weights + pv_tref(m, PV_T_ATTN_NORM, l).off), w.h, d, (float)f.rms_eps);
        PV_HIP(hipGetLastError());
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WQ, l), w.h, nullptr, w.q, rows, s)) != PV_OK) return rc;
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WK, l), w.h, nullptr, w.k, rows, s)) != PV_OK) return rc;
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WV, l), w.h, nullptr, w.v, rows, s)) != PV_OK) return rc;
        if ((rc = pv_k_rope_append(c, l, rows, s)) != PV_OK) return rc;
        k_attention<ST><<<dim3(f.n_q_heads, rows), 256, 0, s>>>(w.state, w.page_table, w.q, (const ST *)c->d_pool, w.attn, g, l, f.n_q_heads);
        PV_HIP(hipGetLastError());
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WO, l), w.attn, w.x, w.x, rows, s)) != PV_OK) return rc;
        k_rmsnorm<ST><<<rows, 256, 0, s>>>(w.x, (const ST *)(m->d_weights + pv_tref(m, PV_T_FFN_NORM, l).off), w.h, d, (float)f.rms_eps);
        PV_HIP(hipGetLastError());
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WG, l), w.h, nullptr, w.gate, rows, s)) != PV_OK) return rc;
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WU, l), w.h, nullptr, w.up, rows, s)) != PV_OK) return rc;
        const size_t nact = (size_t)rows * F;
        k_swiglu<<<(unsigned)((nact + 255) / 256), 256, 0, s>>>(w.gate, w.up, w.gate, nact);
        PV_HIP(hipGetLastError());
        if ((rc = launch_linear<ST>(m, pv_tref(m, PV_T_WD, l), w.gate, w.x, w.x, rows, s)) != PV_OK) return rc;
    }
    const bool head = c->io->hdr[3] != PV_MODE_PREFILL_MID;
    if (head) {
        k_rmsnorm<ST><<<rows, 256, 0, s>>>(w.x, (const ST *)(m->d_weights + m->global[PV_T_FINAL_NORM].off), w.h, d, (float)f.rms_eps);
        PV_HIP(hipGetLastError());
        if ((rc = launch_linear<ST>(m, m->global[PV_T_LM_HEAD], w.h, nullptr, w.logits, rows, s)) != PV_OK) return rc;
    }
    (void)qd;
    if (head && (rc = pv_k_argmax(c, rows, s)) != PV_OK) return rc;
    return pv_k_finish(c, rows, nullptr, nullptr, 0, s);
}

int pv_vec_run_block(pv_cache *c, hipStream_t s)
{
    return c->m->cfg.dtype == PV_BF16 ? run_block<uint16_t>(c, s) : run_block<float>(c, s);
}
