// Matrix-core kernel family for bf16 models.
//
// Skinny GEMMs y[rows<=64][N] = x[rows][K] W^T stream W once from HBM.  W is stored pre-tiled
// in MFMA operand order: strips of 16 output features, each strip a run of K/32 tiles of
// 16x32 bf16 (1 KiB), a tile laid out [lane 0..63][8 bf16] so that one 16-byte load per lane
// is exactly the A operand of v_mfma_f32_16x16x32_bf16.  Up to 16 rows (k_gemm): a workgroup
// owns one or a few strips, its wavefronts split K, accumulate in fp32, and are summed in wave
// order through LDS, so the owner sees complete outputs and the whole epilogue (RMSNorm scale,
// rotary embedding + KV append, SwiGLU, residual add, vocabulary arg-max) is fused into the
// GEMM.  17..64 rows (k_gemm_tile; with 4-bit weights k_gemm_tile_q4, from 9 rows on): the waves
// of a workgroup own different strips, walk K together and share the activation tiles through LDS.
//
// Activations enter as the B operand.  To keep fp32-grade accuracy with bf16 matrix cores an
// activation a is carried as two bf16 numbers hi = bf16(a), lo = bf16(a - hi) (16 mantissa
// bits).  For rows <= 8 the 16 operand columns hold hi of row j in column j and lo in column
// j+8 (rows <= 4: j+4, and the loads mirror columns 4..7 into 8..11: half the bytes), so one
// MFMA does both and the epilogue adds the two column halves; for 9..16 rows hi
// and lo are separate operands and two MFMAs accumulate into the same registers.
//
// RMSNorm is folded in: the producer of x writes (gain * x) as the next operand plus per-strip
// partial sums of x^2; the consumer multiplies its outputs by rsqrt(mean + eps), which
// commutes with the contraction.  Rows of W_q/W_k are permuted inside each head so that the two
// members of a rotary pair sit in the same half of a strip, 4 rows apart (lanes l and l^16 of
// the accumulator; either 8-row half of a strip holds 4 whole pairs); gate and up rows are
// interleaved the same way for SwiGLU (4 gate + 4 up features per half strip).
#include <stdio.h>
#include <stdlib.h>
#include <type_traits>
#include "pv_gemm_epilogue.h"



struct mat_ws {                 // carved out of pv_ws::part
    uint16_t *xop_a, *xop_o, *xop_f, *xop_d;   // operands: QKV in (K=d), O in (K=qd), gate/up in (K=d), down in (K=F)
    float *ssq0, *ssq1;                         // [column tile][d/16][16] partial sums of x^2
    float *pmax_val; int32_t *pmax_idx;         // [row][vocab/16] per-strip arg-max candidates, row-major
    float *attn_part;                           // attention chunk partials
    float *tile_part;                           // K-slice partial sums of the wide-block GEMMs (TILE_PART_FLOATS)
};

static inline size_t xop_elems(int K) { return (size_t)2 * (K / 32) * 512; }   // hi and lo arrays of one 16-row column tile
static inline int col_tiles(int rows) { return rows <= 16 ? 1 : rows <= 32 ? 2 : 4; }
// K-slice partial sums of the shared-tile GEMMs: slices x strips x column tiles KiB.  The launches cut a GEMM of fewer than
// 192 workgroups into at most 16 slices and about 256 workgroups in all, which bounds slices x strips by 16 x 256 + 16 x 191
// (16 strips per workgroup; fewer with 8), i.e. under 2 Mi floats per column tile; 24 MiB in all, which the launches stay under.
static const size_t TILE_PART_FLOATS = (size_t)6 << 20;
static inline size_t tile_part_floats(int col_tiles) { return std::min(TILE_PART_FLOATS, (size_t)col_tiles << 21); }
// blocks that use those kernels: more than 16 rows, or any block of more than 8 rows with 4-bit weights
static inline bool tile_part_needed(const pv_model *m, int col_tiles) { return col_tiles >= 2 || m->wbits == 4; }

static size_t mat_ws_layout(const pv_model *m, int rows_cap, int units_cap, int max_tokens, float *base, mat_ws *w)
{
    const pv_model_config &f = m->cfg;
    const int qd = f.n_q_heads * f.head_dim;
    const size_t ctc = col_tiles(rows_cap);          // every per-row piece is sized for the widest block
    size_t off = 0;   // in floats, every piece a multiple of 64 floats (256 B)
    auto take = [&](size_t floats) { size_t o = off; off += (floats + 63) / 64 * 64; return base ? base + o : (float *)nullptr; };
    float *p;
    p = take(ctc * xop_elems(f.d_model) / 2); if (w) w->xop_a = (uint16_t *)p;
    p = take(ctc * xop_elems(qd) / 2); if (w) w->xop_o = (uint16_t *)p;
    p = take(ctc * xop_elems(f.d_model) / 2); if (w) w->xop_f = (uint16_t *)p;
    p = take(ctc * xop_elems(f.ffn_dim) / 2); if (w) w->xop_d = (uint16_t *)p;
    p = take(ctc * (size_t)f.d_model); if (w) w->ssq0 = p;
    p = take(ctc * (size_t)f.d_model); if (w) w->ssq1 = p;
    p = take(ctc * (size_t)f.vocab); if (w) w->pmax_val = p;
    p = take(ctc * (size_t)f.vocab); if (w) w->pmax_idx = (int32_t *)p;
    p = take(pv_attn_part_floats(m, units_cap, max_tokens)); if (w) w->attn_part = p;
    const size_t tp = tile_part_needed(m, (int)ctc) ? tile_part_floats((int)ctc) : 0;
    p = take(tp); if (w) w->tile_part = tp ? p : nullptr;  // (none: the launches then do not slice)
    return off;
}

size_t pv_mat_part_floats(const pv_model *m, int rows_cap, int units_cap, int max_tokens) { return mat_ws_layout(m, rows_cap, units_cap, max_tokens, nullptr, nullptr); }

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
        strip = h * (head_dim / 16) + p / 8; i = (p & 3) + 4 * side + 8 * ((p >> 2) & 1);
    } else if (perm == PERM_GATEUP) {
        strip = n / 8; i = (int)(n & 3) + 4 * strip_add + 8 * (int)((n >> 2) & 1);   // strip_add: 0 = gate, 1 = up
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

// Rows of a 4-bit matrix, row-major in staging (codes: K/8 dwords per row, a dword = 8 consecutive
// k, low nibble first; scales: K/32 bf16 per row), into the batched strip layout (pv_internal.h).
// One thread moves one dword of codes; the thread of a tile's first dword also moves its scale.
__global__ void k_repack_q4(const uint32_t *codes, const uint16_t *scales, char *dst, int64_t row_begin, int64_t row_count,
                            int K, int perm, int head_dim, int strip_mul, int strip_add)
{
    const int kd = K / 8, nb4 = K / 128;
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= row_count * kd) return;
    const int64_t nl = idx / kd, n = row_begin + nl;
    const int w = (int)(idx % kd), kt = w >> 2, q = w & 3;      // tile, feature-of-k group
    int64_t strip; int i;
    if (perm == PERM_ROPE) {
        const int half = head_dim / 2, e = (int)(n % head_dim);
        const int64_t h = n / head_dim;
        const int side = e >= half, p = e - side * half;
        strip = h * (head_dim / 16) + p / 8; i = (p & 3) + 4 * side + 8 * ((p >> 2) & 1);
    } else if (perm == PERM_GATEUP) {
        strip = n / 8; i = (int)(n & 3) + 4 * strip_add + 8 * (int)((n >> 2) & 1);
    } else {
        strip = (n / 16) * strip_mul + strip_add; i = (int)(n & 15);
    }
    char *batch = dst + ((size_t)strip * nb4 + (kt >> 2)) * PV_Q4_BATCH;
    const int u = kt & 3;
    // the lane's 8 codes c0..c7 (source: c0 in the lowest nibble) are stored as
    // (c0 | c2 << 4 | c4 << 8 | c6 << 12) | (c1 | c3 << 4 | c5 << 8 | c7 << 12) << 16,
    // so that one shift and one mask give the bf16 pair (k = 2t, 2t + 1) of operand dword t
    const uint32_t src = codes[idx];
    uint32_t even = 0, odd = 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) { even |= ((src >> (8 * t)) & 0xFu) << (4 * t); odd |= ((src >> (8 * t + 4)) & 0xFu) << (4 * t); }
    ((uint32_t *)batch)[(i + 16 * q) * 4 + u] = even | (odd << 16);
    if (q == 0) ((uint16_t *)(batch + 1024))[i * 4 + u] = scales[nl * (K / 32) + kt];
}

int pv_mat_repack_q4(const pv_model *m, const pv_tensor_ref &t, int kind, int64_t row_begin, int64_t row_count, size_t scales_off, hipStream_t s)
{
    int perm = PERM_NONE, mul = 1, add = 0;
    if (kind == PV_T_WQ || kind == PV_T_WK) perm = PERM_ROPE;
    else if (kind == PV_T_WG || kind == PV_T_WU) { perm = PERM_GATEUP; add = t.strip_add; }
    const int64_t n = row_count * (t.cols / 8);
    k_repack_q4<<<(unsigned)((n + 255) / 256), 256, 0, s>>>((const uint32_t *)m->d_staging, (const uint16_t *)(m->d_staging + scales_off),
                                                            m->d_weights + t.off, row_begin, row_count, (int)t.cols, perm, m->cfg.head_dim, mul, add);
    PV_HIP(hipGetLastError());
    return PV_OK;
}

// Block set-up on the matrix path: embedding rows -> x, first operand, first sum of squares;
// rotary table for positions len .. len+rows-1.  The draft ids come straight from the cache's
// pinned host mailbox; the first workgroup copies them, the row count and the mode into the
// device state for the kernels that follow.
template <int NB>
__global__ void __launch_bounds__(64)
k_mat_begin(pv_dev_state *st, const int32_t *mailbox, int rows, int mode, const uint16_t *embed, const uint16_t *gain, const double *inv_freq,
            float *x, float *ssq, uint16_t *xop, float2 *rope, int d, int half)
{
    const int lane = threadIdx.x, ct = blockIdx.y, j = ct * 16 + (lane & 15), g = lane >> 4, strip = blockIdx.x;
    const int nseq = st->blk.n_seq;
    const bool tree = mode == PV_MODE_TREE;
    __shared__ int parent[PV_MAX_ROWS];               // draft tree: the parents follow the draft ids in the mailbox; one read each, then walked in LDS
    if (tree) { parent[lane] = lane < rows ? mailbox[PV_MAX_ROWS + lane] : -1; __syncthreads(); }
    // Cache slot of block row r: the cache's length + r, or in a batched step the length of the row's
    // sequence + the row's index inside that sequence's block.  Its rotary position is the same, except in a
    // draft tree, where a row sits at (length + its depth) whatever slot it is stored in.
    auto seq_of = [&](int r) { int sidx = 0; for (int k = 1; k < nseq; ++k) if (r >= st->blk.seq[k].row0) sidx = k; return sidx; };
    auto slot_of = [&](int r) { if (nseq <= 1) return st->len + r; const pv_seq_ref &sq = st->blk.seq[seq_of(r)]; return sq.st->len + r - sq.row0; };
    auto depth_of = [&](int r) { int dpt = 0; for (int q = parent[r]; q >= 0 && dpt < PV_MAX_ROWS; q = parent[q]) ++dpt; return dpt; };
    if (blockIdx.x == 0 && ct == 0) {
        for (int i = lane; i < rows; i += 64) {
            st->draft[i] = mailbox[i]; st->rowseq[i] = nseq <= 1 ? 0 : seq_of(i); st->rowpos[i] = slot_of(i);
            uint64_t m;
            if (tree) { m = 1ull << i; for (int q = parent[i], k = 0; q >= 0 && k < PV_MAX_ROWS; q = parent[q], ++k) m |= 1ull << q; st->parent[i] = parent[i]; }
            else { const int jj = i - (nseq <= 1 ? 0 : st->blk.seq[seq_of(i)].row0); m = jj >= 63 ? ~0ull : (2ull << jj) - 1; }
            st->rowmask[i] = m;
        }
        if (lane == 0) { st->gamma = rows; st->mode = mode; if (nseq <= 1) st->blk.seq[0].gamma = rows; }
    }
    float v[4] = {0.f, 0.f, 0.f, 0.f};
    if (j < rows) {
        const uint16_t *e = embed + (size_t)mailbox[j] * d + strip * 16 + 4 * g;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = pv_bf16_to_f32(e[r]);
    }
    emit_x<NB>(lane, rows, strip, d, v, *(const uint2 *)(gain + strip * 16 + 4 * g), x, ssq, xop, ct, pv_lo_off(rows));
    if (ct != 0) return;
    for (int idx = blockIdx.x * 64 + lane; idx < rows * half; idx += gridDim.x * 64) {
        const int jj = idx / half, i = idx - jj * half;
        double sn, cs;
        sincos((double)(tree ? st->len + depth_of(jj) : slot_of(jj)) * inv_freq[i], &sn, &cs);
        rope[idx] = make_float2((float)cs, (float)sn);
    }
}

// A wave's K walk with DEPTH register buffers: while one batch is used, the loads of the next
// DEPTH - 1 are in flight.  issue(q, k) starts the loads of the wave's k-th batch into q,
// consume(q) uses it; between() runs once behind the first loads (work that may wait on older,
// shorter loads).  Buffers rotate by name, so the steady state is unrolled DEPTH times and every
// issue in it is unconditional: the wait before a consume then only covers that batch's loads.
template <int DEPTH, typename Q, typename FI, typename FC, typename FB>
__device__ inline void k_walk(int cnt, Q &q0, Q &q1, Q &q2, FI issue, FC consume, FB between)
{
    if (cnt > 0) issue(q0, 0);
    if (DEPTH == 3 && cnt > 1) issue(q1, 1);
    between();
    int i = 0;
    if constexpr (DEPTH == 3) {
        for (; i + 4 < cnt; i += 3) {                // q0 and q1 hold batches i and i + 1, in flight or landed
            issue(q2, i + 2); consume(q0);
            issue(q0, i + 3); consume(q1);
            issue(q1, i + 4); consume(q2);
        }
        if (i + 2 < cnt) issue(q2, i + 2);            // at most four batches are left
        if (i < cnt) consume(q0);
        if (i + 3 < cnt) issue(q0, i + 3);
        if (i + 1 < cnt) consume(q1);
        if (i + 2 < cnt) consume(q2);
        if (i + 3 < cnt) consume(q0);
    } else {
        for (; i + 2 < cnt; i += 2) {                // q0 holds batch i
            issue(q1, i + 1); consume(q0);
            issue(q0, i + 2); consume(q1);
        }
        if (i + 1 < cnt) issue(q1, i + 1);            // at most two batches are left
        if (i < cnt) consume(q0);
        if (i + 1 < cnt) consume(q1);
    }
}

// ------------------------------------------------------------------------------------------
// The streaming GEMM: a workgroup owns S adjacent strips, its NW waves split K in batches of U
// tiles.
//
// Rows: NB == 1 packs up to 8 rows (hi and lo halves in one operand; CT == 1).  NB == 2 takes
// the rows in CT column tiles of 16, each with a hi and a lo operand, and keeps S x CT
// accumulators: every operand tile fetched from L2 is used for S strips from registers, which
// keeps the operand traffic (2 CT tiles per batch tile) from outgrowing the weight stream
// (S tiles) in the CU's load path.  (CT > 1 is only used for a K too short for k_gemm_tile.)
//
// K assignment: contiguous runs of batches per wave, or batch b to wave b % NW (the workgroup
// then reads its strips as advancing windows).
// ------------------------------------------------------------------------------------------
//
// DP > 1 (16-bit weights, one column tile): the wave keeps DP batches in registers and loads
// ahead (k_walk): bytes in flight come from depth per wave rather than from the number of
// resident waves.  HF: the last of the S strips is an 8-feature half (see below).
//
// WB == 4: the strip is a run of batches of 4-bit codes and bf16 group scales (one scale per
// output feature and K-tile); the wave walks them with k_walk, two or three batches deep.  A
// code c enters the matrix core as the bf16 number 16 + c (the nibble OR-ed into the top
// mantissa bits of 16.0 = 0x4180: exact).  Per K-tile the accumulator is started by the product
// of the activation tile with an all -24 operand (= -24 x row sums, shared by the S strips), so
// that the codes' product on top of it is sum_k (c_k - 8) * x_k; the vector ALU only multiplies
// that by the tile's scale and adds.  The product is taken transposed (activation rows x
// features) so that a lane's four results share one feature, hence one scale; the accumulators
// are turned back on their way through the LDS reduction.
template <int NB, int CT, int S, int EPI, int NW, int WB = 16, int DP = 1, bool HF = false>
__global__ void __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu((NB == 1 && S == 1 && WB == 16 && DP == 1) ? 8 : (S * CT >= 16) ? 2 : 4)))   // packed bf16 rows, one strip: <= 64 VGPRs, two 16-wave workgroups per CU; 16 accumulator tiles (wide blocks with a short K): more than 128
k_gemm(const gemm_args a)
{
    static_assert(NB == 2 || CT == 1, "packed rows come in one tile");
    static_assert(S <= NW, "one epilogue wave per strip");
    static_assert(WB == 16 || (WB == 4 && CT == 1), "4-bit weights: one column tile");
    static_assert(!HF || ((WB == 4 || DP > 1) && S >= 2), "half strips: walked batches");
    constexpr int U = (S * CT >= 16) ? 1 : (S * CT >= 4) ? 2 : (DP > 1 && (S >= 2 || NB == 2)) ? 2 : 4;   // tiles per batch (16-bit weights)
    constexpr bool NORM = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD);
    constexpr bool PARK = (CT == 1);                 // epilogue inputs fetched early (by the wave that will run the strip's epilogue) and parked in LDS
    // HF: the workgroup owns S - 1 whole strips and one 8-feature half of a strip it shares with
    // its neighbour (strips a.half_base ...), so that a GEMM with (k + 1/2) x 256 strips puts the
    // same bytes on every CU; the lanes of the other half duplicate the owned half's loads for
    // that slot and their rows of the product are not stored.
    const int strip0 = blockIdx.x * (HF ? S - 1 : S), wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int hstrip = HF ? a.half_base + ((int)blockIdx.x >> 1) : 0, hsel = blockIdx.x & 1;
    const int hl = HF ? ((lane & ~8) | (hsel << 3)) - lane : 0;    // half slot: the lanes of the other half read the owned half's lines again (no further bytes)
    const int KT = a.ktiles, nbat = KT / U;        // whole batches of U tiles; a ragged rest goes to the last wave
    int b, bend, bstep;
    if (a.interleave) { b = wave; bend = nbat; bstep = NW; }
    else { const int per = (nbat + NW - 1) / NW; b = min(nbat, wave * per); bend = min(nbat, b + per); bstep = 1; }
    const size_t arr = (size_t)KT * 64;             // tiles of one strip = elements of one operand array, in uint4
    const uint4 *A = a.W + (size_t)strip0 * arr + lane;
    // tile ct: hi at B + (2 ct) arr, lo at B + (2 ct + 1) arr   (NB == 2).  Packed rows of a block of at most 4: hi and lo sit in
    // columns 0..3 and 4..7 of a tile; the lanes of columns 8..11 read the lo columns again, so that the epilogue finds them
    // where a block of 8 has them, and those of 12..15 anything in the same 128-byte line (their columns are never used): half the lines
    int bl = lane;
    if (NB == 1 && a.lo_off == 4) { const int col = lane & 15; bl = (lane & ~15) | (col < 8 ? col : col < 12 ? col - 4 : col - 8); }
    const uint4 *B = a.xop + bl;
    // a ragged last workgroup re-reads its first strip for the missing ones and drops the result
    size_t so[S];
#pragma unroll
    for (int si = 0; si < S; ++si) so[si] = (HF && si == S - 1) ? (size_t)(hstrip - strip0) * arr : (strip0 + si < a.nstrips) ? (size_t)si * arr : 0;
    f32x4 acc[S][CT];
#pragma unroll
    for (int si = 0; si < S; ++si)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[si][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

    __shared__ f32x4 red[NW][S][CT][64];
    __shared__ float ssq_s[NW][CT][16];
    __shared__ epi_pre pre_s[PARK ? S : 1][PARK ? 64 : 1];

    // RMSNorm of the input rows: every wave takes its share of the per-strip sums of squares; the
    // loads go out ahead of the weight stream and are folded in behind its first batch
    ssq_loads<(WB == 4 && NW <= 8) ? 16 / NW * 2 : 2> sl[CT];   // d up to 8192 without a serial tail of loads
    if (NORM) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) ssq_issue(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl[ct]);
    }

    const size_t qstrip = (size_t)(KT / 4) * PV_Q4_BATCH;
    const char *Aq = (const char *)a.W + (size_t)strip0 * qstrip;
    if constexpr (WB == 4) {
        // One batch = 4 K-tiles.  A wave keeps three batches in registers: while one is used the
        // loads of the next two are in flight, so that the wave always has bytes on the way.
        // The product is taken transposed here (activation rows x features): all four results
        // of a lane then belong to one feature, and the lane needs one scale per tile.
        struct qbatch { uint4 c[S]; uint2 s[S]; uint4 bh[4], bl[NB == 2 ? 4 : 1]; };
        const int nb4 = KT >> 2, wv = __builtin_amdgcn_readfirstlane(wave);    // batch addresses in scalar registers
        int first, cnt, bstride;
        if (a.interleave) { first = wv; bstride = NW; cnt = wv < nb4 ? (nb4 - wv + NW - 1) / NW : 0; }
        else { const int per = (nb4 + NW - 1) / NW; first = min(nb4, wv * per); cnt = min(nb4, first + per) - first; bstride = 1; }
        size_t qo[S];
#pragma unroll
        for (int si = 0; si < S; ++si) qo[si] = (HF && si == S - 1) ? (size_t)(hstrip - strip0) * qstrip : (strip0 + si < a.nstrips) ? (size_t)si * qstrip : 0;
        auto issue = [&](qbatch &q, int k) {          // k-th batch of this wave
            const int bt = first + k * bstride;
#pragma unroll
            for (int si = 0; si < S; ++si) {
                const char *p = Aq + qo[si] + (size_t)bt * PV_Q4_BATCH;
                const int ln = lane + ((HF && si == S - 1) ? hl : 0);
                q.c[si] = load_once((const uint4 *)(p + ln * 16));
                q.s[si] = load_once((const uint2 *)(p + 1024 + (ln & 15) * 8));
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const size_t o = (size_t)(bt * 4 + u) * 64;
                q.bh[u] = B[o];
                if (NB == 2) q.bl[NB == 2 ? u : 0] = B[arr + o];
            }
            asm volatile("" ::: "memory");           // the loads go out here, ahead of the arithmetic that follows
        };
        // -24 in every element: its product with the activation tile starts the accumulator at
        // -24 x (row sums), on top of which the codes' product lands as sum (c - 8) x
        const uint4 neg24 = make_uint4(0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u);
        auto consume = [&](const qbatch &q) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                f32x4 T0 = {0.f, 0.f, 0.f, 0.f};
                T0 = mfma16(q.bh[u], neg24, T0);
                if (NB == 2) T0 = mfma16(q.bl[NB == 2 ? u : 0], neg24, T0);
#pragma unroll
                for (int si = 0; si < S; ++si) {
                    const uint4 c4 = q.c[si];
                    const uint32_t cw = u == 0 ? c4.x : u == 1 ? c4.y : u == 2 ? c4.z : c4.w;
                    const uint32_t sw = (u & 2) ? q.s[si].y : q.s[si].x;
                    const float sc = __uint_as_float((u & 1) ? (sw & 0xFFFF0000u) : (sw << 16));
                    // operand dword t = bf16 pair (16 + c_2t, 16 + c_2t+1): nibble t of each half into the top mantissa bits of 16.0
                    const uint4 wa = make_uint4(((cw << 3) & 0x00780078u) | 0x41804180u, ((cw >> 1) & 0x00780078u) | 0x41804180u,
                                                ((cw >> 5) & 0x00780078u) | 0x41804180u, ((cw >> 9) & 0x00780078u) | 0x41804180u);
                    f32x4 T = mfma16(q.bh[u], wa, T0);
                    if (NB == 2) T = mfma16(q.bl[NB == 2 ? u : 0], wa, T);
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[si][0][r] = fmaf(sc, T[r], acc[si][0][r]);
                }
            }
        };
        constexpr int DEPTH = (NB == 2 || S >= 3) ? 2 : 3;   // what fits in 128 registers
        qbatch q0, q1, q2;
        k_walk<DEPTH>(cnt, q0, q1, q2, issue, consume, [&]() {
            if (NORM) {
                const float4 s4 = ssq_finish(a.ssq, a.ssq_parts, threadIdx.x, NW * 64, sl[0]);
                if (lane < 4) *(float4 *)&ssq_s[wave][0][4 * lane] = s4;
            }
            if (PARK && wave < S) {
                epi_pre pre;
                epi_prefetch<EPI>(a, (HF && wave == S - 1) ? hstrip : min(strip0 + wave, a.nstrips - 1), lane, pre, 0);
                epi_park<EPI>(&pre_s[wave][lane], pre);
            }
        });
        // acc is (row 4 g + r, feature f) for lane (g, f); the sum below and the epilogues take
        // (feature 4 g' + r', row j) from lane (g', j): store transposed
        {
            float *rf = (float *)&red[wave][0][0][0];
            const int g = lane >> 4, f = lane & 15;
#pragma unroll
            for (int si = 0; si < S; ++si)
#pragma unroll
                for (int r = 0; r < 4; ++r) rf[si * 256 + ((f >> 2) * 16 + 4 * g + r) * 4 + (f & 3)] = acc[si][0][r];
        }
    } else if constexpr (DP > 1) {
        static_assert(CT == 1, "deep variant: one column tile");
        struct wbatch { uint4 w[S][U], x[U], xl[NB == 2 ? U : 1]; };     // xl: the lo halves of a 16-row tile
        const int wv = __builtin_amdgcn_readfirstlane(wave);
        int first, cnt, bstride;
        if (a.interleave) { first = wv; bstride = NW; cnt = wv < nbat ? (nbat - wv + NW - 1) / NW : 0; }
        else { const int per = (nbat + NW - 1) / NW; first = min(nbat, wv * per); cnt = min(nbat, first + per) - first; bstride = 1; }
        auto issue = [&](wbatch &q, int k) {
            const size_t o = (size_t)(first + k * bstride) * U * 64;
#pragma unroll
            for (int u = 0; u < U; ++u) {
#pragma unroll
                for (int si = 0; si < S; ++si) q.w[si][u] = load_once(&A[so[si] + o + u * 64 + ((HF && si == S - 1) ? hl : 0)]);
                q.x[u] = B[o + u * 64];
                if (NB == 2) q.xl[NB == 2 ? u : 0] = B[arr + o + u * 64];
            }
            asm volatile("" ::: "memory");
        };
        auto consume = [&](const wbatch &q) {
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int si = 0; si < S; ++si) {
                    acc[si][0] = mfma16(q.w[si][u], q.x[u], acc[si][0]);
                    if (NB == 2) acc[si][0] = mfma16(q.w[si][u], q.xl[NB == 2 ? u : 0], acc[si][0]);
                }
        };
        wbatch q0, q1, q2;
        k_walk<DP>(cnt, q0, q1, q2, issue, consume, [&]() {
            if (NORM) {
                const float4 s4 = ssq_finish(a.ssq, a.ssq_parts, threadIdx.x, NW * 64, sl[0]);
                if (lane < 4) *(float4 *)&ssq_s[wave][0][4 * lane] = s4;
            }
            if (PARK && wave < S) {
                epi_pre pre;
                epi_prefetch<EPI>(a, (HF && wave == S - 1) ? hstrip : min(strip0 + wave, a.nstrips - 1), lane, pre, 0);
                epi_park<EPI>(&pre_s[wave][lane], pre);
            }
        });
        if (wave == NW - 1) {
            for (int t = nbat * U; t < KT; ++t) {
                const uint4 x = B[(size_t)t * 64];
                uint4 xl = x;
                if (NB == 2) xl = B[arr + (size_t)t * 64];
#pragma unroll
                for (int si = 0; si < S; ++si) {
                    const uint4 w = load_once(&A[so[si] + (size_t)t * 64 + ((HF && si == S - 1) ? hl : 0)]);
                    acc[si][0] = mfma16(w, x, acc[si][0]);
                    if (NB == 2) acc[si][0] = mfma16(w, xl, acc[si][0]);
                }
            }
        }
    } else {
    uint4 ra[S][U], rb[CT][U], rc[CT][U];
    auto load_batch = [&](int t) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t o = (size_t)(t + u) * 64;
#pragma unroll
            for (int si = 0; si < S; ++si) ra[si][u] = load_once(&A[so[si] + o]);
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                rb[ct][u] = B[(size_t)(2 * ct) * arr + o];
                if (NB == 2) rc[ct][u] = B[(size_t)(2 * ct + 1) * arr + o];
            }
        }
    };
    auto use_batch = [&]() {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int si = 0; si < S; ++si)
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    acc[si][ct] = mfma16(ra[si][u], rb[ct][u], acc[si][ct]);
                    if (NB == 2) acc[si][ct] = mfma16(ra[si][u], rc[ct][u], acc[si][ct]);
                }
    };

    // Few registers on purpose (NB == 1): latency is hidden by many resident waves per CU.
    {   // first batch peeled: the sums of squares are folded in while its loads are in flight
        const bool first = b < bend;
        if (first) load_batch(b * U);
        if (NORM) {
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const float4 s4 = ssq_finish(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl[ct]);
                if (lane < 4) *(float4 *)&ssq_s[wave][ct][4 * lane] = s4;
            }
        }
        if (PARK && wave < S) {                     // behind the first batch's loads, ahead of its use
            epi_pre pre;
            epi_prefetch<EPI>(a, min(strip0 + wave, a.nstrips - 1), lane, pre, 0);
            epi_park<EPI>(&pre_s[wave][lane], pre);
        }
        if (first) { use_batch(); b += bstep; }
    }
    for (; b < bend; b += bstep) {
        load_batch(b * U);
        use_batch();
    }
    if (wave == NW - 1) {

        for (int t = nbat * U; t < KT; ++t) {
            const size_t o = (size_t)t * 64;
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) {
                const uint4 bh = B[(size_t)(2 * ct) * arr + o];
                uint4 bl = bh;
                if (NB == 2) bl = B[(size_t)(2 * ct + 1) * arr + o];
#pragma unroll
                for (int si = 0; si < S; ++si) {
                    const uint4 wa = load_once(&A[so[si] + o]);
                    acc[si][ct] = mfma16(wa, bh, acc[si][ct]);
                    if (NB == 2) acc[si][ct] = mfma16(wa, bl, acc[si][ct]);
                }
            }
        }
    }
    }   // WB == 16

    // sum the NW K-slices (and the NW shares of the sums of squares) in wave order; wave si runs
    // the epilogue of strip strip0 + si
    if (WB == 16) {
#pragma unroll
        for (int si = 0; si < S; ++si)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct) red[wave][si][ct][lane] = acc[si][ct];
    }
    __syncthreads();
    const bool hslot = HF && wave == S - 1;
    if (wave >= S || (!hslot && strip0 + wave >= a.nstrips)) return;
    const int strip = hslot ? hstrip : strip0 + wave;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) {
        f32x4 sum = red[0][wave][ct][lane];
        for (int w = 1; w < NW; ++w) { const f32x4 p = red[w][wave][ct][lane]; sum[0] += p[0]; sum[1] += p[1]; sum[2] += p[2]; sum[3] += p[3]; }
        epi_pre pre;
        if (PARK) epi_unpark<EPI>(&pre_s[wave][lane], pre);
        else epi_prefetch<EPI>(a, strip, lane, pre, ct);
        if (NORM) {
            float tot = ssq_s[0][ct][lane & 15];
#pragma unroll
            for (int w = 1; w < NW; ++w) tot += ssq_s[w][ct][lane & 15];
            pre.rj = 1.0f / sqrtf(tot * a.inv_d + a.eps);
        }
        if (hslot && (lane >> 5) != hsel) pre.rows = 0;           // features 4 (lane / 16) .. + 3 of the other half: nothing to store
        epi_apply<NB, EPI>(a, strip, lane, sum, pre, ct);
    }
}

// ------------------------------------------------------------------------------------------
// Blocks of 17..64 rows (CT = 2 or 4 column tiles of 16 rows, a hi and a lo operand each): 2 CT
// activation tiles go with every weight tile.  Fetched per wave they outgrow the weight stream
// in the CU's load path, so here the 8 waves of a workgroup walk the same K range in step, each
// with its own S strips, and every activation tile is fetched once per workgroup and shared
// through LDS (two buffers, one barrier per step of U K-tiles).  Weights and activation tiles
// are loaded D steps ahead into registers; the activation tiles pass through LDS on use.
// A GEMM with few strips is cut along K as well (blockIdx.y): the slices' partial sums go to
// `part` and k_tile_finish adds them in slice order and runs the epilogue; with one slice the
// epilogue runs here.  Workgroups start their K walk at different steps so that they do not
// all stream from addresses a power of two apart.
// ------------------------------------------------------------------------------------------
template <int CT, int S, int EPI>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(4)))
k_gemm_tile(const gemm_args a, int tps, float4 *part)
{
    constexpr int NW = 8, U = 2, D = 4, TPS = U * CT * 2, NLD = TPS / NW;    // TPS activation tiles per step, NLD of them per wave
    static_assert((NLD == 1 || (NLD == 2 && CT * 2 == NW)) && TPS == NLD * NW, "a wave loads one tile of the step, or two of the same operand array");
    constexpr bool NORM = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int KT = a.ktiles, t0 = blockIdx.y * tps, t1 = min(KT, t0 + tps);  // this slice's K-tiles (not empty: the launch sees to it)
    const int nsteps = (t1 - t0 + U - 1) / U;
    const int rot = (int)((blockIdx.x * 5u + blockIdx.y * 3u) % (unsigned)nsteps);
    const size_t arr = (size_t)KT * 64;
    const int sw = (blockIdx.x * NW + wave) * S;                              // the wave's first strip
    size_t so[S];                                                             // strips past the end re-read the last one; dropped below
#pragma unroll
    for (int si = 0; si < S; ++si) so[si] = (size_t)min(sw + si, a.nstrips - 1) * arr;
    const uint4 *A = a.W + lane, *B = a.xop + lane;
    __shared__ uint4 sa[2][TPS][64];
    __shared__ float ssq_s[NW][CT][16];

    ssq_loads<2> sl[CT];
    if (NORM && part == nullptr) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) ssq_issue(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl[ct]);
    }
    f32x4 acc[S][CT];
#pragma unroll
    for (int si = 0; si < S; ++si)
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) acc[si][ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

    struct slot { uint4 x0, x1, w[S][U]; };           // one step in flight: the wave's one or two activation tiles, its weight tiles
    auto first_tile = [&](int step) { int k = step + rot; if (k >= nsteps) k -= nsteps; return t0 + k * U; };
    auto issue = [&](slot &q, int step) {             // loads of (rotated) step `step`; a tile past the slice's end re-reads its last one
        const int tb = first_tile(step);
        {   // tile t of the step: K-tile t / (2 CT) of it, operand array t % (2 CT); the wave takes tiles wave and wave + 8
            const int u = wave / (CT * 2), r = wave % (CT * 2);
            q.x0 = B[(size_t)r * arr + (size_t)min(tb + u, t1 - 1) * 64];
            if (NLD == 2) q.x1 = B[(size_t)r * arr + (size_t)min(tb + u + 1, t1 - 1) * 64];   // CT = 4: 8 more tiles = the next K-tile, same array
        }
#pragma unroll
        for (int si = 0; si < S; ++si)
#pragma unroll
            for (int u = 0; u < U; ++u) q.w[si][u] = load_once(&A[so[si] + (size_t)min(tb + u, t1 - 1) * 64]);
        asm volatile("" ::: "memory");
    };
    auto use = [&](const slot &q, int buf, int step) {   // q holds step `step`: share its activation tiles through sa[buf], multiply
        sa[buf][wave][lane] = make_uint4(q.x0.x, q.x0.y, q.x0.z, q.x0.w);
        if (NLD == 2) sa[buf][wave + NW][lane] = make_uint4(q.x1.x, q.x1.y, q.x1.z, q.x1.w);
        __syncthreads();
        const int tb = first_tile(step);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (tb + u < t1) {
#pragma unroll
                for (int ct = 0; ct < CT; ++ct) {
                    const uint4 hi = sa[buf][u * CT * 2 + 2 * ct][lane], lo = sa[buf][u * CT * 2 + 2 * ct + 1][lane];
#pragma unroll
                    for (int si = 0; si < S; ++si) {
                        acc[si][ct] = mfma16(q.w[si][u], hi, acc[si][ct]);
                        acc[si][ct] = mfma16(q.w[si][u], lo, acc[si][ct]);
                    }
                }
            }
        }
    };
    static_assert(D == 4, "slots are spelled out");
    slot q0, q1, q2, q3;
    issue(q0, 0);
    issue(q1, min(1, nsteps - 1));
    issue(q2, min(2, nsteps - 1));
    issue(q3, min(3, nsteps - 1));
    if (NORM && part == nullptr) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const float4 s4 = ssq_finish(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl[ct]);
            if (lane < 4) *(float4 *)&ssq_s[wave][ct][4 * lane] = s4;
        }
    }
    int s0 = 0;
    for (; s0 + D <= nsteps; s0 += D) {               // every wave of the workgroup takes the same steps: the barriers match
        use(q0, 0, s0);     issue(q0, min(s0 + 4, nsteps - 1));
        use(q1, 1, s0 + 1); issue(q1, min(s0 + 5, nsteps - 1));
        use(q2, 0, s0 + 2); issue(q2, min(s0 + 6, nsteps - 1));
        use(q3, 1, s0 + 3); issue(q3, min(s0 + 7, nsteps - 1));
    }
    if (s0 < nsteps) use(q0, 0, s0);
    if (s0 + 1 < nsteps) use(q1, 1, s0 + 1);
    if (s0 + 2 < nsteps) use(q2, 0, s0 + 2);

    if (part != nullptr) {
#pragma unroll
        for (int si = 0; si < S; ++si)
#pragma unroll
            for (int ct = 0; ct < CT; ++ct)
                if (sw + si < a.nstrips) part[(((size_t)blockIdx.y * a.nstrips + sw + si) * CT + ct) * 64 + lane] = make_float4(acc[si][ct][0], acc[si][ct][1], acc[si][ct][2], acc[si][ct][3]);
        return;
    }
    __syncthreads();                                  // (ssq_s of every wave; also covers a slice of a single step)
#pragma unroll
    for (int si = 0; si < S; ++si) {
        const int strip = sw + si;
        if (strip >= a.nstrips) continue;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            epi_pre pre;
            epi_prefetch<EPI>(a, strip, lane, pre, ct);
            if (NORM) {
                float tot = ssq_s[0][ct][lane & 15];
#pragma unroll
                for (int w = 1; w < NW; ++w) tot += ssq_s[w][ct][lane & 15];
                pre.rj = 1.0f / sqrtf(tot * a.inv_d + a.eps);
            }
            epi_apply<2, EPI>(a, strip, lane, acc[si][ct], pre, ct);
        }
    }
}

// ------------------------------------------------------------------------------------------
// The same for 4-bit weights (9..64 rows, CT = 1, 2 or 4): the 8 waves of a workgroup own two strips each and walk
// the strips' batches (4 K-tiles of codes + scales, 1152 bytes) in step; the 8 CT activation tiles of
// a step are fetched once per workgroup and shared through LDS (two buffers, one barrier per step).
// Per weight byte a 4-bit strip needs 3.6 times the activation bytes of a 16-bit one, on the L2 -> CU
// path as well as out of LDS: hence two strips per wave.  A step is long (72 MFMAs at 64 rows), so the
// weights are loaded two steps ahead and the activation tiles one (their registers are free once they sit in LDS).
// Arithmetic as in k_gemm<WB = 4>: a code c enters as the bf16 number 16 + c, the product is taken
// transposed (activation rows x features) on top of -24 x (row sums), scaled per K-tile; the row sums
// are the same for every strip and are taken once per workgroup by the wave that brings the tile in.
// The accumulators are turned back through LDS before the epilogue (or before they are stored as a
// K-slice's partial sums for k_tile_finish).
// ------------------------------------------------------------------------------------------
template <int CT, int EPI>
__global__ void __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_gemm_tile_q4(const gemm_args a, int bps, float4 *part)
{
    constexpr int NW = 8, S = 2, U = 4, P = U * CT, TPS = P * 2;            // P (K-tile, column tile) pairs = TPS activation tiles per step
    static_assert(CT == 1 || CT == 2 || CT == 4, "a wave brings in pair `wave` (if there is one) and, with 16 pairs, pair `wave + 8`");
    constexpr bool NORM = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD);
    extern __shared__ uint4 tile_lds[];                         // [2][TPS][64]
    uint4 (*sa)[TPS][64] = (uint4 (*)[TPS][64])tile_lds;
    __shared__ float ssq_s[NW][CT][16];
    __shared__ f32x4 rs[2][TPS / 2][4];                         // per (K-tile, column tile) of a step: -24 x its rows' sums, rows 4 g .. 4 g + 3 at [g]
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int NBAT = a.ktiles >> 2;                             // batches of a strip
    const int b0 = blockIdx.y * bps, b1 = min(NBAT, b0 + bps), nsteps = b1 - b0;   // this slice (not empty: the launch sees to it)
    const int rot = (int)((blockIdx.x * 5u + blockIdx.y * 3u) % (unsigned)nsteps);
    const size_t arr = (size_t)a.ktiles * 64;
    const int sw = (blockIdx.x * NW + wave) * S;                // the wave's first strip; strips past the end: the last one again, dropped below
    const char *Aq0 = (const char *)a.W + (size_t)min(sw, a.nstrips - 1) * (size_t)NBAT * PV_Q4_BATCH;
    const char *Aq1 = (const char *)a.W + (size_t)min(sw + 1, a.nstrips - 1) * (size_t)NBAT * PV_Q4_BATCH;
    const uint4 *B = a.xop + lane;

    ssq_loads<2> sl[CT];
    if (NORM && part == nullptr) {
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) ssq_issue(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl[ct]);
    }
    f32x4 acc0[CT], acc1[CT];
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) acc0[ct] = acc1[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};

    struct wslot { uint4 c0, c1; uint2 s0, s1; };               // a batch of either strip
    struct xslot { uint4 a, b, c, d; };                         // (named members: an array here ends up in scratch memory)
    const bool loads = wave < P;                                // (CT = 1: four pairs a step, the other four waves bring in none)
    auto batch_of = [&](int step) { int k = min(step, nsteps - 1) + rot; if (k >= nsteps) k -= nsteps; return b0 + k; };   // (a step past the end re-reads the last one)
    auto issue_w = [&](wslot &q, int step) {
        const size_t o = (size_t)batch_of(step) * PV_Q4_BATCH;
        q.c0 = load_once((const uint4 *)(Aq0 + o + lane * 16));
        q.c1 = load_once((const uint4 *)(Aq1 + o + lane * 16));
        q.s0 = load_once((const uint2 *)(Aq0 + o + 1024 + (lane & 15) * 8));
        q.s1 = load_once((const uint2 *)(Aq1 + o + 1024 + (lane & 15) * 8));
        asm volatile("" ::: "memory");
    };
    auto issue_x = [&](xslot &q, int step) {                    // pair p = wave (+ 8) of the step: K-tile p / CT of the batch, column tile p % CT, hi and lo
        const int bt = batch_of(step);
        auto tile = [&](int p, int half) { const int u = p / CT, ct = p % CT; return B[(size_t)(2 * ct + half) * arr + (size_t)(bt * 4 + u) * 64]; };
        if (loads) { q.a = tile(wave, 0); q.b = tile(wave, 1); }
        if (P > NW) { q.c = tile(wave + NW, 0); q.d = tile(wave + NW, 1); }
        asm volatile("" ::: "memory");
    };
    const uint4 neg24 = make_uint4(0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u, 0xC1C0C1C0u);
    auto stage = [&](const xslot &x, int buf) {                 // the wave's tiles of the step into LDS, with -24 x the row sums of each hi + lo pair
        const f32x4 zero4 = {0.f, 0.f, 0.f, 0.f};
        if (loads) {
            sa[buf][2 * wave][lane] = x.a; sa[buf][2 * wave + 1][lane] = x.b;
            const f32x4 ra = mfma16(x.b, neg24, mfma16(x.a, neg24, zero4));
            if ((lane & 15) == 0) rs[buf][wave][lane >> 4] = ra;
        }
        if (P > NW) {
            sa[buf][2 * (wave + NW)][lane] = x.c; sa[buf][2 * (wave + NW) + 1][lane] = x.d;
            const f32x4 rc = mfma16(x.d, neg24, mfma16(x.c, neg24, zero4));
            if ((lane & 15) == 0) rs[buf][wave + NW][lane >> 4] = rc;
        }
    };
    uint32_t sixteen = 0x41804180u;                             // (in a vector register, so that mask-and-merge is one instruction)
    asm volatile("" : "+v"(sixteen));
    auto codes = [&](uint32_t cw) {                             // 8 codes of a dword as the bf16 numbers 16 + c, in operand order
        auto pick = [&](uint32_t v) { uint32_t r; asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(v), "s"(0x00780078u), "v"(sixteen)); return r; };
        return make_uint4(pick(cw << 3), pick(cw >> 1), pick(cw >> 5), pick(cw >> 9));
    };
    auto scale = [](uint2 s2, int u) { const uint32_t w = (u & 2) ? s2.y : s2.x; return __uint_as_float((u & 1) ? (w & 0xFFFF0000u) : (w << 16)); };
    // One (K-tile, column tile) pair after the other, software-pipelined by hand: the LDS reads of the next pair go out,
    // then the four MFMAs of this pair, then the scaling of the previous pair's products (whose MFMAs are done by then);
    // the scheduling fences keep that order, which the compiler would otherwise serialise (read, wait, multiply, wait, scale).
    auto compute = [&](const wslot &w, int buf) {
        uint4 hiN = sa[buf][0][lane], loN = sa[buf][1][lane], wa0, wa1;
        f32x4 t0N = rs[buf][0][lane >> 4], pa, pb;
        float sc0 = 0.f, sc1 = 0.f, ps0 = 0.f, ps1 = 0.f;
#pragma unroll
        for (int p = 0; p < U * CT; ++p) {
            const int u = p / CT, ct = p % CT;
            const uint4 hi = hiN, lo = loN;
            const f32x4 T0 = t0N;
            if (ct == 0) {
                wa0 = codes(u == 0 ? w.c0.x : u == 1 ? w.c0.y : u == 2 ? w.c0.z : w.c0.w);
                wa1 = codes(u == 0 ? w.c1.x : u == 1 ? w.c1.y : u == 2 ? w.c1.z : w.c1.w);
                sc0 = scale(w.s0, u); sc1 = scale(w.s1, u);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (p + 1 < U * CT) { hiN = sa[buf][2 * p + 2][lane]; loN = sa[buf][2 * p + 3][lane]; t0N = rs[buf][p + 1][lane >> 4]; }
            __builtin_amdgcn_sched_barrier(0);
            f32x4 Ta = mfma16(hi, wa0, T0), Tb = mfma16(hi, wa1, T0);
            Ta = mfma16(lo, wa0, Ta); Tb = mfma16(lo, wa1, Tb);
            __builtin_amdgcn_sched_barrier(0);
            if (p > 0) {
                const int pc = (p - 1) % CT;
#pragma unroll
                for (int r = 0; r < 4; ++r) { acc0[pc][r] = fmaf(ps0, pa[r], acc0[pc][r]); acc1[pc][r] = fmaf(ps1, pb[r], acc1[pc][r]); }
            }
            pa = Ta; pb = Tb; ps0 = sc0; ps1 = sc1;
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) { acc0[CT - 1][r] = fmaf(ps0, pa[r], acc0[CT - 1][r]); acc1[CT - 1][r] = fmaf(ps1, pb[r], acc1[CT - 1][r]); }
    };
    wslot wA, wB;
    xslot x = {};
    issue_w(wA, 0); issue_w(wB, 1);
    if (NORM && part == nullptr) {                              // (their loads went out before the weights': no wait for those; the
#pragma unroll                                                  //  registers are free again before the activation slot fills)
        for (int ct = 0; ct < CT; ++ct) {
            const float4 s4 = ssq_finish(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl[ct]);
            if (lane < 4) *(float4 *)&ssq_s[wave][ct][4 * lane] = s4;
        }
    }
    issue_x(x, 0);
    // every wave of the workgroup takes the same steps: the barriers match.  Buffer i & 1 is rewritten at step i + 2,
    // behind the barrier of step i + 1, which every wave reaches with its reads of step i done.
#define PV_Q4_STEP(W, I)                                                                     \
    if (s0 + (I) < nsteps) { stage(x, (I) & 1); issue_x(x, s0 + (I) + 1); __syncthreads(); compute(W, (I) & 1); issue_w(W, s0 + (I) + 2); }
    for (int s0 = 0; s0 < nsteps; s0 += 2) { PV_Q4_STEP(wA, 0) PV_Q4_STEP(wB, 1) }
#undef PV_Q4_STEP
    __syncthreads();                                            // the last step's tiles have been read; ssq_s of every wave
    // an accumulator is (row 4 g + r, feature f) for lane (g, f); the epilogues take (feature 4 g' + r', row j) from
    // lane (g', j): turned through the wave's own KiB of the tile buffer
    float *rf = (float *)&sa[0][wave][0];
    const int g = lane >> 4, f = lane & 15;
    auto turn = [&](f32x4 &v) {
#pragma unroll
        for (int r = 0; r < 4; ++r) rf[((f >> 2) * 16 + 4 * g + r) * 4 + (f & 3)] = v[r];
        const f32x4 t = ((const f32x4 *)rf)[lane];              // (a wave's LDS traffic stays in order: no barrier inside the wave)
        v = t;
    };
#pragma unroll
    for (int ct = 0; ct < CT; ++ct) { turn(acc0[ct]); turn(acc1[ct]); }
#pragma unroll
    for (int si = 0; si < S; ++si) {
        const int strip = sw + si;
        if (strip >= a.nstrips) continue;
#pragma unroll
        for (int ct = 0; ct < CT; ++ct) {
            const f32x4 v = si == 0 ? acc0[ct] : acc1[ct];
            if (part != nullptr) {
                part[(((size_t)blockIdx.y * a.nstrips + strip) * CT + ct) * 64 + lane] = make_float4(v[0], v[1], v[2], v[3]);
                continue;
            }
            epi_pre pre;
            epi_prefetch<EPI>(a, strip, lane, pre, ct);
            if (NORM) {
                float tot = ssq_s[0][ct][lane & 15];
#pragma unroll
                for (int w = 1; w < NW; ++w) tot += ssq_s[w][ct][lane & 15];
                pre.rj = 1.0f / sqrtf(tot * a.inv_d + a.eps);
            }
            epi_apply<2, EPI>(a, strip, lane, v, pre, ct);
        }
    }
}

// Adds the K-slices' partial sums of k_gemm_tile in slice order and runs the epilogue: one wave
// per (strip, column tile), the four waves of a workgroup take four strips of column tile
// blockIdx.y.  At most TILE_MAX_SLICES slices: their loads go out together.
#define TILE_MAX_SLICES 16
template <int CT, int EPI>
__global__ void __launch_bounds__(256)
k_tile_finish(const gemm_args a, const float4 *part, int slices)
{
    constexpr int NW = 4;
    constexpr bool NORM = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LMHEAD);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, ct = blockIdx.y;
    const int strip = min((int)blockIdx.x * NW + wave, a.nstrips - 1);           // a wave past the end repeats the last strip's loads and stores nothing
    const bool mine = (int)blockIdx.x * NW + wave < a.nstrips;
    __shared__ float ssq_s[NW][16];
    ssq_loads<4> sl;
    if (NORM) ssq_issue(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl);
    float4 p[TILE_MAX_SLICES];
#pragma unroll
    for (int y = 0; y < TILE_MAX_SLICES; ++y) p[y] = part[(((size_t)(y < slices ? y : 0) * a.nstrips + strip) * CT + ct) * 64 + lane];
    epi_pre pre;
    epi_prefetch<EPI>(a, strip, lane, pre, ct);
    if (NORM) {
        const float4 s4 = ssq_finish(a.ssq + (size_t)ct * a.ssq_parts * 16, a.ssq_parts, threadIdx.x, NW * 64, sl);
        if (lane < 4) *(float4 *)&ssq_s[wave][4 * lane] = s4;
        __syncthreads();
        float tot = ssq_s[0][lane & 15];
#pragma unroll
        for (int w = 1; w < NW; ++w) tot += ssq_s[w][lane & 15];
        pre.rj = 1.0f / sqrtf(tot * a.inv_d + a.eps);
    }
    float4 v = p[0];
#pragma unroll
    for (int y = 1; y < TILE_MAX_SLICES; ++y)
        if (y < slices) { v.x += p[y].x; v.y += p[y].y; v.z += p[y].z; v.w += p[y].w; }
    if (mine) epi_apply<2, EPI>(a, strip, lane, (f32x4){v.x, v.y, v.z, v.w}, pre, ct);   // (wave-uniform; no barrier inside)
}

// ------------------------------- host side ----------------------------------------



static constexpr size_t tile_q4_lds(int ct) { return (size_t)2 * 4 * ct * 2 * 64 * sizeof(uint4); }   // two buffers of 8 ct activation tiles

template <int CT, int EPI>
static int allow_tile_q4_lds()
{
    PV_HIP(hipFuncSetAttribute((const void *)k_gemm_tile_q4<CT, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)tile_q4_lds(CT)));
    return PV_OK;
}

// once per device before the first launch (and outside any stream capture): the wide-block kernels for 4-bit
// weights use more dynamic LDS than the default limit
int pv_mat_gemm_init(void)
{
    int rc;
    if ((rc = allow_tile_q4_lds<1, EPI_QKV>()) != PV_OK || (rc = allow_tile_q4_lds<1, EPI_RESID>()) != PV_OK ||
        (rc = allow_tile_q4_lds<1, EPI_SWIGLU>()) != PV_OK || (rc = allow_tile_q4_lds<1, EPI_LMHEAD>()) != PV_OK ||
        (rc = allow_tile_q4_lds<2, EPI_QKV>()) != PV_OK || (rc = allow_tile_q4_lds<2, EPI_RESID>()) != PV_OK ||
        (rc = allow_tile_q4_lds<2, EPI_SWIGLU>()) != PV_OK || (rc = allow_tile_q4_lds<2, EPI_LMHEAD>()) != PV_OK ||
        (rc = allow_tile_q4_lds<4, EPI_QKV>()) != PV_OK || (rc = allow_tile_q4_lds<4, EPI_RESID>()) != PV_OK ||
        (rc = allow_tile_q4_lds<4, EPI_SWIGLU>()) != PV_OK || (rc = allow_tile_q4_lds<4, EPI_LMHEAD>()) != PV_OK) return rc;
    return PV_OK;
}

template <int NB, int CT, int EPI>
static int launch_gemm(const pv_model *m, const gemm_args &g, int strips, hipStream_t s)
{
    gemm_args ga = g;
    ga.nstrips = strips;
    ga.interleave = g.ktiles > 128;                          // long strips: measured 0.3 % faster per step, short ones 0.3 % slower
    if (m->wbits == 4) {
        if constexpr (NB == 1) {
            // Several strips per workgroup share every activation tile from registers (one strip:
            // 4 KiB of tiles from L2 per 1.1 KiB of weights), as many as still leave a workgroup per CU.
            if constexpr (EPI == EPI_QKV || EPI == EPI_SWIGLU) {
                // strips = (k + 1/2) x G with G a multiple of the 256 CUs: G workgroups of k whole strips and
                // half of a shared one put the same bytes on every CU (see the 16-bit launch below)
                for (int k = (strips >= 1024 ? 3 : 2); k >= 1 && g.ktiles >= 64; --k) {
                    const int G = 2 * strips / (2 * k + 1);
                    if (2 * strips % (2 * k + 1) != 0 || G % 256 != 0 || G == 0) continue;
                    ga.half_base = k * G;
                    if (k == 3) k_gemm<1, 1, 4, EPI, 8, 4, 1, true><<<G, 512, 0, s>>>(ga);
                    else if (k == 2) k_gemm<1, 1, 3, EPI, 8, 4, 1, true><<<G, 512, 0, s>>>(ga);
                    else k_gemm<1, 1, 2, EPI, 8, 4, 1, true><<<G, 512, 0, s>>>(ga);
                    PV_HIP(hipGetLastError());
                    return PV_OK;
                }
            }
            if (strips >= 1024 && g.ktiles >= 64) k_gemm<1, 1, 4, EPI, 8, 4><<<(strips + 3) / 4, 512, 0, s>>>(ga);
            else if (strips >= 512 && g.ktiles >= 64) k_gemm<1, 1, 2, EPI, 8, 4><<<(strips + 1) / 2, 512, 0, s>>>(ga);
            else if (g.ktiles >= 64) k_gemm<1, 1, 1, EPI, 16, 4><<<strips, 1024, 0, s>>>(ga);
            else k_gemm<1, 1, 1, EPI, 8, 4><<<strips, 512, 0, s>>>(ga);
        } else {
            // 4-bit weights, 9..64 rows: activation tiles shared through LDS, two strips per wave, one workgroup per CU
            // (256 registers a lane); few strips: cut along K so that about 256 workgroups run, as for 16-bit weights
            const int nbat = g.ktiles / 4, ngroups = (strips + 15) / 16;
            int slices = (ngroups >= 192 || g.tile_part == nullptr) ? 1 : min(TILE_MAX_SLICES, (256 + ngroups - 1) / ngroups);
            int bps = max(4, (nbat + slices - 1) / slices);
            slices = (nbat + bps - 1) / bps;
            while (slices > 1 && (size_t)slices * strips * CT * 256 > tile_part_floats(CT)) { bps += 1; slices = (nbat + bps - 1) / bps; }
            float4 *part = slices > 1 ? (float4 *)g.tile_part : nullptr;
            k_gemm_tile_q4<CT, EPI><<<dim3(ngroups, slices), 512, tile_q4_lds(CT), s>>>(ga, bps, part);
            PV_HIP(hipGetLastError());
            if (slices > 1) { k_tile_finish<CT, EPI><<<dim3((strips + 3) / 4, CT), 256, 0, s>>>(ga, part, slices); PV_HIP(hipGetLastError()); }
            return PV_OK;
        }
    } else if constexpr (NB == 2) {
        // Strips per workgroup: with enough strips to fill the machine anyway, the 2 CT operand
        // tiles per batch tile are matched by as many weight tiles (S = 2 or 4); a GEMM with few
        // strips keeps one strip per workgroup and more waves instead.
        constexpr int S = CT == 1 ? 2 : 4, NW = CT == 1 ? 8 : 4;
        if constexpr (CT >= 2) {
            // activation tiles shared through LDS; few strips: cut along K so that about 256 workgroups run
            if (g.ktiles >= 16) {
                const int ngroups = (strips + 7) / 8;
                int slices = (ngroups >= 192 || g.tile_part == nullptr) ? 1 : min(TILE_MAX_SLICES, (256 + ngroups - 1) / ngroups);
                int tps = (g.ktiles + slices - 1) / slices;
                tps = max(8, (tps + 1) & ~1);                        // whole steps, at least four per slice
                slices = (g.ktiles + tps - 1) / tps;
                while (slices > 1 && (size_t)slices * strips * CT * 256 > tile_part_floats(CT)) { tps += 2; slices = (g.ktiles + tps - 1) / tps; }
                float4 *part = slices > 1 ? (float4 *)g.tile_part : nullptr;
                k_gemm_tile<CT, 1, EPI><<<dim3(ngroups, slices), 512, 0, s>>>(ga, tps, part);
                PV_HIP(hipGetLastError());
                if (slices > 1) { k_tile_finish<CT, EPI><<<dim3((strips + 3) / 4, CT), 256, 0, s>>>(ga, part, slices); PV_HIP(hipGetLastError()); }
                return PV_OK;
            }
        }
        if constexpr (CT == 1) {
            // one column tile: batches walked several deep, like the packed rows (measured 2 - 3 % per step)
            if (g.ktiles >= 64) {
                bool done = false;
                if constexpr (EPI == EPI_QKV) {       // (k + 1/2) x 256 strips: half strips as for the packed rows
                    if (strips % 256 == 128 && strips / 256 >= 1 && strips / 256 <= 2) {
                        ga.half_base = (strips / 256) * 256;
                        if (strips / 256 == 1) k_gemm<NB, CT, 2, EPI, 8, 16, 3, true><<<256, 512, 0, s>>>(ga);
                        else k_gemm<NB, CT, 3, EPI, 8, 16, 2, true><<<256, 512, 0, s>>>(ga);
                        done = true;
                    }
                }
                if (done) ;
                else if (strips >= 512) k_gemm<NB, CT, 2, EPI, 8, 16, 2><<<(strips + 1) / 2, 512, 0, s>>>(ga);
                else k_gemm<NB, CT, 1, EPI, 8, 16, 3><<<strips, 512, 0, s>>>(ga);
                PV_HIP(hipGetLastError());
                return PV_OK;
            }
        }
        if (strips >= 256 * S) k_gemm<NB, CT, S, EPI, NW><<<(strips + S - 1) / S, NW * 64, 0, s>>>(ga);
        else if (CT == 1 && g.ktiles >= 64) k_gemm<NB, CT, 1, EPI, 16><<<strips, 1024, 0, s>>>(ga);
        else k_gemm<NB, CT, 1, EPI, 8><<<strips, 512, 0, s>>>(ga);
    } else {
        // Eight waves, each three batches deep (two workgroups per CU at <= 128 registers): measured
        // 1 - 8 % faster per GEMM than sixteen waves that load and use one batch at a time; a short K
        // has too few batches per wave for that
        // Two strips per workgroup share every activation tile; taken where the halved number of
        // workgroups fills the 256 CUs as evenly as the full one (measured, 70B shapes: gate/up
        // 165 -> 156 us, down 79 -> 75 us, vocabulary projection 97 -> 92 us; where it would leave
        // CUs unevenly loaded, e.g. 640 or 1792 strips, one strip per workgroup is 3 - 10 % faster)
        // (k + 1/2) x 256 strips (the fused QKV projection of both benchmark shapes): k whole strips
        // and half of a shared one per workgroup, 256 workgroups
        if constexpr (EPI == EPI_QKV) {
            if (g.ktiles >= 64 && strips % 256 == 128 && strips / 256 >= 1 && strips / 256 <= 2) {
                ga.half_base = (strips / 256) * 256;
                if (strips / 256 == 1) k_gemm<NB, CT, 2, EPI, 8, 16, 3, true><<<256, 512, 0, s>>>(ga);
                else k_gemm<NB, CT, 3, EPI, 8, 16, 2, true><<<256, 512, 0, s>>>(ga);
                PV_HIP(hipGetLastError());
                return PV_OK;
            }
        }
        if constexpr (EPI == EPI_SWIGLU) {
            // 3.5 x G strips, G a multiple of the CUs: three whole strips and a half per workgroup, so that every CU holds
            // the same number of equal workgroups from start to end (70B-shaped gate/up: 156.5 -> 153.7 us; 8B-shaped, 1792
            // strips, which one strip per workgroup spreads as seven per CU, two at a time: 44.0 -> 41.5 us)
            if (g.ktiles >= 128 && (2 * strips) % 7 == 0 && (2 * strips / 7) % 256 == 0) {
                const int G = 2 * strips / 7;
                ga.half_base = 3 * G;
                k_gemm<NB, CT, 4, EPI, 8, 16, 2, true><<<G, 512, 0, s>>>(ga);
                PV_HIP(hipGetLastError());
                return PV_OK;
            }
        }
        auto fill = [](int wgs) { return (double)wgs / (double)(((wgs + 255) / 256) * 256); };
        const bool two = strips >= 512 && fill((strips + 1) / 2) >= fill(strips);
        if (g.ktiles >= 64 && two) k_gemm<NB, CT, 2, EPI, 8, 16, 2><<<(strips + 1) / 2, 512, 0, s>>>(ga);
        else if (g.ktiles >= 64) k_gemm<NB, CT, 1, EPI, 8, 16, 3><<<strips, 512, 0, s>>>(ga);
        else k_gemm<NB, CT, 1, EPI, 8><<<strips, 512, 0, s>>>(ga);
    }
    PV_HIP(hipGetLastError());
    return PV_OK;
}

template <int NB, int CT>
static int run_block(pv_cache *c, hipStream_t s)
{
    const pv_model *m = c->m;
    const pv_model_config &f = m->cfg;
    const int rows = c->last_rows, d = f.d_model, hd = f.head_dim, qd = f.n_q_heads * hd, kvd = f.n_kv_heads * hd, F = f.ffn_dim;
    mat_ws mw;
    mat_ws_layout(m, c->rows_cap, c->units_cap, c->n_pages * f.page_tokens, c->ws.part, &mw);
    const char *Wb = m->d_weights;
    auto gainp = [&](int kind, int l) { return (const uint16_t *)(Wb + pv_tref(m, kind, l).off); };

    k_mat_begin<NB><<<dim3(d / 16, CT), 64, 0, s>>>(c->ws.state, c->d_io->draft, rows, c->io->hdr[3], (const uint16_t *)(Wb + m->global[PV_T_EMBED].off), gainp(PV_T_ATTN_NORM, 0),
                                           (const double *)(Wb + m->inv_freq_off), c->ws.x, mw.ssq0, mw.xop_a, c->ws.rope, d, hd / 2);
    PV_HIP(hipGetLastError());

    gemm_args g = {};
    int prc;
    g.st = c->ws.state; g.lo_off = pv_lo_off(rows); g.inv_d = 1.0f / (float)d; g.eps = (float)f.rms_eps; g.ssq_parts = d / 16;
    g.q_hi = (uint16_t *)c->ws.q; g.q_lo = g.q_hi + (size_t)c->rows_cap * qd; g.pool = (uint16_t *)c->d_pool; g.page_table = c->ws.page_table; g.rope = c->ws.rope; g.geom = pv_geom(c);
    g.n_q_heads = f.n_q_heads; g.q_strips = qd / 16; g.k_strips = kvd / 16;
    g.x = c->ws.x; g.d = d; g.xop_act = mw.xop_d; g.F = F;
    g.logits = c->ws.logits; g.pmax_val = mw.pmax_val; g.pmax_idx = mw.pmax_idx; g.vocab = f.vocab;
    g.tile_part = mw.tile_part;

    for (int l = 0; l < f.n_layers; ++l) {
        // fused QKV projection: RMSNorm scale, rotary embedding, KV append
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WQ, l).off); g.xop = (const uint4 *)mw.xop_a; g.ktiles = d / 32;
        g.ssq = mw.ssq0; g.layer = l;
        if ((prc = pv_prof_mark(c, PV_PROF_QKV, l, 0, s)) != PV_OK) return prc;
        if ((prc = launch_gemm<NB, CT, EPI_QKV>(m, g, (qd + 2 * kvd) / 16, s)) != PV_OK) return prc;
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
        if ((prc = launch_gemm<NB, CT, EPI_RESID>(m, g, d / 16, s)) != PV_OK) return prc;
        if ((prc = pv_prof_mark(c, PV_PROF_OPROJ, l, 1, s)) != PV_OK) return prc;
        // gate/up projection + SwiGLU
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WG, l).off); g.xop = (const uint4 *)mw.xop_f; g.ktiles = d / 32;
        g.ssq = mw.ssq1;
        if ((prc = pv_prof_mark(c, PV_PROF_GATEUP, l, 0, s)) != PV_OK) return prc;
        if ((prc = launch_gemm<NB, CT, EPI_SWIGLU>(m, g, F / 8, s)) != PV_OK) return prc;
        if ((prc = pv_prof_mark(c, PV_PROF_GATEUP, l, 1, s)) != PV_OK) return prc;
        // down projection + residual; emits the next layer's (or the head's) operand
        g.W = (const uint4 *)(Wb + pv_tref(m, PV_T_WD, l).off); g.xop = (const uint4 *)mw.xop_d; g.ktiles = F / 32;
        g.gain_next = (l + 1 < f.n_layers) ? gainp(PV_T_ATTN_NORM, l + 1) : (const uint16_t *)(Wb + m->global[PV_T_FINAL_NORM].off);
        g.ssq_out = mw.ssq0; g.xop_out = mw.xop_a;
        if ((prc = pv_prof_mark(c, PV_PROF_DOWN, l, 0, s)) != PV_OK) return prc;
        if ((prc = launch_gemm<NB, CT, EPI_RESID>(m, g, d / 16, s)) != PV_OK) return prc;
        if ((prc = pv_prof_mark(c, PV_PROF_DOWN, l, 1, s)) != PV_OK) return prc;
    }
    const bool head = c->io->hdr[3] != PV_MODE_PREFILL_MID;
    if (head) {
        g.W = (const uint4 *)(Wb + m->global[PV_T_LM_HEAD].off); g.xop = (const uint4 *)mw.xop_a; g.ktiles = d / 32; g.ssq = mw.ssq0;
        if ((prc = pv_prof_mark(c, PV_PROF_LMHEAD, 0, 0, s)) != PV_OK) return prc;
        if ((prc = launch_gemm<NB, CT, EPI_LMHEAD>(m, g, f.vocab / 16, s)) != PV_OK) return prc;
        if ((prc = pv_prof_mark(c, PV_PROF_LMHEAD, 0, 1, s)) != PV_OK) return prc;
    }
    return pv_k_finish(c, rows, mw.pmax_val, mw.pmax_idx, f.vocab / 16, s);
}

int pv_mat_run_block(pv_cache *c, hipStream_t s)
{
    const int rows = c->last_rows;
    if (rows > 64) { pv_set_error("matrix path handles at most 64 rows per block"); return PV_ERANGE; }
    if (rows <= 8) return run_block<1, 1>(c, s);
    if (rows <= 16) return run_block<2, 1>(c, s);
    if (rows <= 32) return run_block<2, 2>(c, s);
    return run_block<2, 4>(c, s);
}
