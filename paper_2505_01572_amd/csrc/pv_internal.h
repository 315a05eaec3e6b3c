// Internal declarations shared by the host API and the two kernel families.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "pipeverify.h"

#define PV_MAX_ROWS 64          // hard cap on rows per block (max_gamma)
#define PV_KEY_BUCKETS 24       // attention grids of recorded steps are sized for the next power of two of (length + rows)
#define PV_ROW_PAD 16           // activation buffers are padded to a multiple of this many rows

// step modes written into pv_dev_state::mode
enum { PV_MODE_VERIFY = 0, PV_MODE_PREFILL_LAST = 1, PV_MODE_PREFILL_MID = 2, PV_MODE_TREE = 3 };
#define PV_N_MODES 4

#define PV_MAX_SEQ 16           // sequences whose blocks one batched step may stack

// One sequence of a block as the kernels see it.  A plain step has one (the cache itself); a batched
// step (pv_verify_batch) stacks the blocks of several caches of one model into one pass over the
// weights: rows row0 .. row0 + gamma - 1 of the stacked block belong to this sequence, their keys and
// values live in this sequence's pages, their positions follow this sequence's length.
struct pv_dev_state;
struct pv_seq_ref {
    pv_dev_state *st;           // the sequence's own state (len, pending; accepted / next_token on return)
    void *pool;                 // its KV pages
    const int32_t *page_table;
    int32_t gamma, row0;
    int32_t n_pages, unit0;     // pool geometry; first attention row-group unit of this sequence
};
struct pv_block_desc {          // which sequences the running block is made of
    int32_t n_seq, pad;
    pv_seq_ref seq[PV_MAX_SEQ];
};

// Per-cache state that lives in device memory so that a step needs no host-side patching:
// every kernel reads the cache length and row count from here.  For a batched step the state of
// the first cache (the "leader") describes the block; len / pending / accepted / next_token stay
// per sequence in each cache's own state.
struct pv_dev_state {
    int32_t len;                // committed tokens
    int32_t pending;            // stage's own prediction for position len, -1 = unknown
    int32_t gamma;              // rows of the running block (all sequences together)
    int32_t mode;
    int32_t accepted, next_token;
    int32_t pad[2];
    int32_t draft[PV_MAX_ROWS];
    int32_t pred[PV_MAX_ROWS];
    int32_t rowseq[PV_MAX_ROWS];    // sequence of each row and the cache slot (absolute position) its K/V go to (written by the block set-up)
    int32_t rowpos[PV_MAX_ROWS];
    uint64_t rowmask[PV_MAX_ROWS];  // which of its sequence's block slots a row may attend to: bit q = the slot at (sequence length + q).
                                    // A chain: slots 0 .. the row's own; a draft tree: the row's ancestors and itself
    int32_t parent[PV_MAX_ROWS];    // draft tree (PV_MODE_TREE): parent row of each row, -1 = a child of the committed prefix
    int32_t path[PV_MAX_ROWS];      // ... and, on return, the rows of the accepted path in order
    pv_block_desc blk;
};

// pinned host mailbox (one per cache)
struct pv_host_io {
    int32_t draft[PV_MAX_ROWS];
    int32_t parent[PV_MAX_ROWS];   // draft tree: parent row of each row
    int32_t hdr[4];             // len, pending, gamma, mode
    int32_t result[2 * PV_MAX_SEQ + 2];   // written by the step's last kernel: (accepted, next_token) per sequence, then the error flag
    pv_block_desc single;       // the one-sequence description of this cache (constant)
    pv_block_desc batch;        // staging of a batched step's description
};
#define PV_RESULT_ERR (2 * PV_MAX_SEQ)

struct pv_tensor_ref {
    size_t  off;                // byte offset in the weight arena
    int64_t rows, cols;
    int64_t loaded_rows;
    // matrix path: 16-row strip i of this tensor is strip (i*strip_mul + strip_add) of the tiled
    // region starting at `off` (gate/up are interleaved strip by strip; q,k,v are concatenated)
    int32_t strip_mul, strip_add;
};

struct pv_model {
    pv_model_config cfg;
    int path;                   // PV_PATH_VECTOR or PV_PATH_MATRIX (resolved)
    int wbits;                  // 16, or 4: projection matrices and LM head as codes + group scales
    int elt;                    // bytes per stored element
    char *d_weights; size_t weight_bytes;
    char *d_staging; size_t staging_bytes;
    pv_tensor_ref *layer;       // [n_layers][PV_T_NKINDS]
    pv_tensor_ref global[PV_T_NKINDS];
    size_t inv_freq_off;        // double[head_dim/2]
    int n_cus;
};

struct pv_ws {                  // pointers into the caller's workspace
    pv_dev_state *state;
    int32_t *page_table;
    float2 *rope;               // [rows][head_dim/2] (cos, sin)
    float *x, *h, *q, *k, *v, *attn, *gate, *up, *logits;
    float *part;                // matrix path: operands, partial sums, attention partials
    size_t part_floats;
};

struct pv_cache {
    const pv_model *m;
    char *d_pool; size_t pool_bytes;
    char *d_ws; size_t ws_bytes;
    int32_t max_tokens, n_pages, rows_cap;
    int32_t units_cap;          // attention row-group units the workspace's partial arrays hold
    pv_ws ws;
    pv_host_io *io;             // pinned host memory, mapped into the device's address space
    pv_host_io *d_io;           // the same mailbox as the kernels address it
    int32_t len, pending, last_rows;
    int32_t blk_start, blk_rows;   // positions the last block wrote K/V for (blk_rows = 0: none on record)
    int32_t attn_keys;          // keys the attention launch of the step being enqueued has to cover (host-side bound: length + rows)
    int32_t blk_units, blk_seq_rows; // batched step in the making: attention row-group units in all, most rows of one sequence (0: plain step)
    bool in_flight; hipStream_t flight_stream;
    // instrumentation: one kernel kind bracketed by events, one pair per layer
    int32_t prof_kind, prof_pending;
    hipEvent_t *prof_ev;        // [2 * n_layers], created on first use
    double prof_ms; int64_t prof_launches;
    // one instantiated HIP graph per (rows, mode) of the step's launch sequence, captured on first use
    bool use_graphs;
    hipStream_t cap_stream;     // private stream that only ever records
    hipGraphExec_t gexec[PV_MAX_ROWS + 1][PV_N_MODES][PV_KEY_BUCKETS];   // ... and per power-of-two bucket of the keys attention covers
};

// bracket helper used by the kernel families: records the start/end event of slot `slot`
// when `kind` is the selected kernel
int pv_prof_mark(pv_cache *c, int kind, int slot, int end, hipStream_t s);

static inline const pv_tensor_ref &pv_tref(const pv_model *m, int kind, int layer)
{
    if (kind == PV_T_EMBED || kind == PV_T_FINAL_NORM || kind == PV_T_LM_HEAD) return m->global[kind];
    return m->layer[(size_t)layer * PV_T_NKINDS + kind];
}

// KV page pool addressing, in elements:
//   block(layer, phys_page, kv_head, which) = (((layer*n_pages + phys)*n_kv_heads + kv_head)*2 + which) * page_tokens*head_dim
// Inside a block, element (token t of the page, feature e):
//   vector path  K: [t][e]                    V: [e][t]            (V transposed inside the page)
//   matrix path  tokens grouped by 16 (one MFMA tile of keys), group s = t/16, u = t%16:
//                K: [s][e/32][u + 16*((e%32)/8)][e%8]   -- each 16x32 sub-tile is an MFMA A operand
//                V: [s][e][u]
struct pv_kv_geom {
    int32_t n_pages, n_kv_heads, page_tokens, head_dim, page_shift, tiled;
};

__host__ __device__ static inline size_t pv_kv_block(const pv_kv_geom &g, int layer, int phys, int kvh, int which)
{
    return ((((size_t)layer * g.n_pages + phys) * g.n_kv_heads + kvh) * 2 + which) * (size_t)(g.page_tokens * g.head_dim);
}

__host__ __device__ static inline size_t pv_k_off(const pv_kv_geom &g, int t, int e)
{
    if (!g.tiled) return (size_t)t * g.head_dim + e;
    return (size_t)(t >> 4) * 16 * g.head_dim + (size_t)(((e >> 5) * 64) + (t & 15) + 16 * ((e & 31) >> 3)) * 8 + (e & 7);
}

__host__ __device__ static inline size_t pv_v_off(const pv_kv_geom &g, int t, int e)
{
    if (!g.tiled) return (size_t)e * g.page_tokens + t;
    return (size_t)(t >> 4) * 16 * g.head_dim + (size_t)e * 16 + (t & 15);
}

// ---- kernel-family entry points (host functions that enqueue on `s`) ----
int pv_vec_run_block(pv_cache *c, hipStream_t s);        // pv_kernels_vector.hip
int pv_mat_run_block(pv_cache *c, hipStream_t s);        // pv_kernels_matrix.hip
int pv_mat_repack(const pv_model *m, const pv_tensor_ref &t, int kind, int64_t row_begin, int64_t row_count, hipStream_t s);
int pv_mat_repack_q4(const pv_model *m, const pv_tensor_ref &t, int kind, int64_t row_begin, int64_t row_count, size_t scales_off, hipStream_t s);

// 4-bit matrices: a strip (16 output features) is a run of cols/128 batches of PV_Q4_BATCH bytes:
// 4 K-tiles of codes, [lane 0..63][tile 0..3] dwords (a dword = the lane's 8 consecutive k of its
// row), then the 64 bf16 scales of the batch as [feature 0..15][tile 0..3].
#define PV_Q4_BATCH 1152
static inline bool pv_is_q4_kind(int kind)
{
    return kind == PV_T_WQ || kind == PV_T_WK || kind == PV_T_WV || kind == PV_T_WO || kind == PV_T_WG || kind == PV_T_WU ||
           kind == PV_T_WD || kind == PV_T_LM_HEAD;
}
size_t pv_mat_part_floats(const pv_model *m, int rows_cap, int units_cap, int max_tokens);
size_t pv_attn_part_floats(const pv_model *m, int units_cap, int max_tokens);
int pv_attn_units(const pv_model *m, int rows);              // attention row-group units of one sequence with `rows` rows
int pv_mat_attention_init(int head_dim);
int pv_mat_gemm_init(void);
int pv_mat_attention(pv_cache *c, int layer, int rows, float *part, uint16_t *xop_o, hipStream_t s);
void pv_set_error(const char *fmt, ...);

#define PV_HIP(call)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) {                                                             \
            pv_set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return PV_EHIP;                                                                 \
        }                                                                                   \
    } while (0)
