/*
 * pipeverify — the verification step of one PipeSpec pipeline stage on one MI355X (gfx950).
 *
 * A stage M_i keeps a key/value cache for the tokens it has committed.  One verify call
 * runs the stage's LLaMA-style decoder over a block of gamma draft tokens appended to that
 * cache, takes the argmax at every position, accepts the longest draft prefix that equals
 * the stage's own greedy decoding, produces one correction token, and rolls the cache back
 * past the first rejection (paper: Sec. 3.2 and Algorithm 1, "verify drafts" branch;
 * Sec. 3.3, text after Eq. 1: a rejecting verifier generates one token itself; Sec. 4.1:
 * greedy decoding).  Rollback requested by a later stage is pv_rollback (Algorithm 1,
 * "rollback O_i to match O_j's last token").
 *
 * Conventions
 *  - Plain C ABI.  Every function returns PV_OK (0) or a negative pv_status; nothing throws
 *    or aborts.  pv_strerror() names a status; pv_last_error() gives the calling thread's
 *    last detailed message.
 *  - "host" pointers are ordinary CPU memory, "device" pointers are HIP device memory on the
 *    current device.  The caller allocates and owns every device buffer (sizes come from
 *    pv_model_bytes / pv_cache_bytes) and must keep it alive, untouched, until the object
 *    using it is destroyed.  The library owns only its small host-side handles and a few
 *    hundred bytes of pinned host memory per cache.
 *  - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls on
 *    one cache must not overlap; different caches (also of one model) may run concurrently
 *    on different streams.
 *  - Tokens are int32 ids in [0, vocab).  Matrices are handed over row-major as
 *    [out_features][in_features] (y = x W^T), in the model's storage type.
 */
#ifndef PIPEVERIFY_H
#define PIPEVERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PV_OK = 0,
    PV_EINVAL = -1,   /* null pointer, bad enum, unsupported shape                        */
    PV_ESTATE = -2,   /* prefix_len != cache length, weights missing, cache not empty ...  */
    PV_ERANGE = -3,   /* gamma > max_gamma, length + gamma > max_tokens, token id outside  */
    PV_EHIP = -4,     /* a HIP runtime call failed (see pv_last_error)                     */
    PV_ENOMEM = -5,   /* a caller-provided buffer is too small / host allocation failed    */
    PV_ENUMERIC = -6  /* a row of the block had no finite logit (NaN weights / activations): the
                         step committed nothing, length and pending are as before the call     */
} pv_status;

typedef enum { PV_F32 = 0, PV_BF16 = 1 } pv_dtype;

/* Tensor kinds for pv_load_weights.  Matrices are [out][in]; norm gains are [1][d_model]. */
typedef enum {
    PV_T_EMBED = 0,      /* [vocab][d_model]                    */
    PV_T_ATTN_NORM = 1,  /* per layer                            */
    PV_T_WQ = 2,         /* [n_q_heads*head_dim][d_model]        */
    PV_T_WK = 3,         /* [n_kv_heads*head_dim][d_model]       */
    PV_T_WV = 4,         /* [n_kv_heads*head_dim][d_model]       */
    PV_T_WO = 5,         /* [d_model][n_q_heads*head_dim]        */
    PV_T_FFN_NORM = 6,
    PV_T_WG = 7,         /* gate  [ffn_dim][d_model]             */
    PV_T_WU = 8,         /* up    [ffn_dim][d_model]             */
    PV_T_WD = 9,         /* down  [d_model][ffn_dim]             */
    PV_T_FINAL_NORM = 10,
    PV_T_LM_HEAD = 11,   /* [vocab][d_model], not tied to EMBED  */
    PV_T_NKINDS = 12
} pv_tensor_kind;

/* Which kernel family runs the step. */
typedef enum {
    PV_PATH_AUTO = 0,    /* PV_F32 -> vector path, PV_BF16 -> matrix-core path            */
    PV_PATH_VECTOR = 1,  /* row-major weights, fp32 vector-ALU kernels (any storage type)  */
    PV_PATH_MATRIX = 2   /* bf16 weights repacked into MFMA tiles, streamed by fused GEMMs */
} pv_kernel_path;

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab;
    double  rms_eps;      /* added to mean(x^2) inside the square root                     */
    double  rope_base;    /* rotary base; rotate-half pairing (i, i + head_dim/2)          */
    int32_t dtype;        /* pv_dtype of weights and of the KV cache                       */
    int32_t page_tokens;  /* tokens per KV page, power of two, >= 16 on the matrix path    */
    int32_t max_gamma;    /* largest block (rows) one verify / prefill chunk may carry, <= 64 */
    int32_t kernel_path;  /* pv_kernel_path                                                */
    int32_t weight_bits;  /* 0 or 16: matrices stored in `dtype`.  4: the projection matrices and
                           * the LM head are 4-bit codes with one bf16 scale per 32 input
                           * features, weight = (code - 8) * scale (the 4-bit target model of the
                           * paper's Sec. 4.1; format chosen by this library); needs PV_BF16, the
                           * matrix path, input widths that are multiples of 128 */
} pv_model_config;

#define PV_Q4_GROUP 32      /* input features per scale of a 4-bit matrix */

typedef struct pv_model pv_model;   /* immutable once all weights are loaded */
typedef struct pv_cache pv_cache;   /* one sequence of one stage             */

/* ---- sizes: the caller allocates all device memory ----
 * (The paper runs stock LLaMA-2 / LLaMA-3 checkpoints, Sec. 4.1, and is silent on memory layout,
 * loading and cache management: everything from here to pv_cache_set_page_table is this library's
 * own design around the public LLaMA decoder definition.) */

/* weight_bytes: device arena for all weights (+ small tables).  staging_bytes: device scratch
 * used only while pv_load_weights runs (may be freed after the last load has completed). */
int pv_model_bytes(const pv_model_config *cfg, size_t *weight_bytes, size_t *staging_bytes);

/* page_pool_bytes: KV pages for max_tokens tokens.  workspace_bytes: activations, partial
 * results, logits of one step. */
int pv_cache_bytes(const pv_model *m, int32_t max_tokens, size_t *page_pool_bytes, size_t *workspace_bytes);

/* ---- objects ---- */

/* d_weights / d_staging: device, 256-byte aligned, at least the sizes reported above. */
int pv_model_create(const pv_model_config *cfg, void *d_weights, size_t weight_bytes,
                    void *d_staging, size_t staging_bytes, pv_model **out);
void pv_model_destroy(pv_model *m);

/*
 * Hand over rows [row_begin, row_begin + row_count) of one tensor (the stage's model M_i of Sec. 3.2;
 * the paper says nothing on how weights reach the device).  host_rows points at the
 * first of those rows (row-major, storage type of the model).  May be called many times per
 * tensor so that the host never holds a whole model; the chunks of a tensor come in row order
 * (row_begin = the end of the previous chunk, or 0 to start the tensor over; anything else is
 * PV_ESTATE) and every tensor must be complete before the first pv_prefill / pv_verify.  On the matrix path row_begin and
 * row_count must be multiples of 16 (except for the norm gains).  The rows are copied to
 * the device and repacked there; the call returns after the copy out of host_rows is done
 * (host_rows may be reused), the repack is ordered on hip_stream.  `layer` is ignored for
 * EMBED / FINAL_NORM / LM_HEAD.
 */
int pv_load_weights(pv_model *m, int32_t kind, int32_t layer, int64_t row_begin, int64_t row_count,
                    const void *host_rows, void *hip_stream);

/* Rows of one matrix of a 4-bit model (kinds WQ, WK, WV, WO, WG, WU, WD, LM_HEAD; every other
 * tensor of such a model goes through pv_load_weights).  host_codes: [row_count][cols / 2] bytes,
 * two codes per byte, the even input feature in the low nibble; host_scales: [row_count][cols /
 * 32] bf16 bit patterns.  Same row, chunk and synchronisation rules as pv_load_weights. */
int pv_load_weights_q4(pv_model *m, int32_t kind, int32_t layer, int64_t row_begin, int64_t row_count,
                       const void *host_codes, const void *host_scales, void *hip_stream);

/* The stage's key/value cache (Sec. 2.1: keys and values of the committed tokens are kept so that a
 * step only computes its new positions), paged.  d_page_pool / d_workspace: device, 256-byte aligned.
 * The new cache is empty (length 0, pending unknown) with the identity page table. */
int pv_cache_create(const pv_model *m, void *d_page_pool, size_t page_pool_bytes,
                    void *d_workspace, size_t workspace_bytes, int32_t max_tokens, pv_cache **out);
void pv_cache_destroy(pv_cache *c);

/* Replace the logical->physical page map (host array, a permutation of 0..n_pages-1 where
 * n_pages = ceil(max_tokens / page_tokens)).  Only on an empty cache (else PV_ESTATE). */
int pv_cache_set_page_table(pv_cache *c, const int32_t *phys_pages, int32_t n_pages, void *hip_stream);

/* ---- the step ---- */

/*
 * The prefill phase of Sec. 2.1 (the prompt is processed in parallel before decoding starts):
 * append n prompt tokens (host array), all accepted, in chunks of at most max_gamma rows
 * (matrix path: of up to 64 rows, whatever max_gamma is).
 * Afterwards length += n and pending = the stage's greedy token after the prompt.
 * Synchronises hip_stream before returning.
 */
int pv_prefill(pv_cache *c, const int32_t *tokens, int32_t n, void *hip_stream);

/*
 * Verify draft[0..gamma) (host array) on top of the cached prefix.
 *   pred[j]     = argmax_v logits(prefix ++ draft[0..j])[v], ties -> lowest id
 *   expected[0] = pending if known, otherwise draft[0] is trusted (always accepted)
 *   expected[j] = pred[j-1] for j >= 1
 *   n           = largest m with draft[j] == expected[j] for all j < m      (0 <= n <= gamma)
 *   next_token  = pred[n-1] if n >= 1, else pending
 * On return *accepted_len = n, *next_token as above (host), the cache holds
 * prefix ++ draft[0..n) (K/V of rejected positions are dead) and pending = next_token.
 * prefix_len is a guard: it must equal the cache length (else PV_ESTATE, nothing changes).
 * gamma = 1 with pending unknown is one plain greedy decoding step (Algorithm 1, stage 0).
 * Synchronises hip_stream before returning.
 */
int pv_verify(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma,
              int32_t *accepted_len, int32_t *next_token, void *hip_stream);

/* Same step without the final wait: results become readable through pv_verify_wait. Between
 * the two calls no other call may touch this cache. */
int pv_verify_async(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma, void *hip_stream);
int pv_verify_wait(pv_cache *c, int32_t *accepted_len, int32_t *next_token);

/*
 * Verify the blocks of several sequences in one pass over the weights (Sec. 2.2: verification pays
 * because the weight and KV-cache loads are shared by all the tokens of a step; stacking the blocks
 * of independent sequences shares the weight loads further).  caches[0..n_seq): distinct caches of
 * one bf16 model on the matrix path, all created with the same max_tokens; sequence i contributes
 * gamma[i] <= max_gamma draft tokens, draft = their concatenation (host arrays), sum of gamma[i] <= 64
 * (<= max_gamma with 4-bit weights), n_seq <= 16.  Every sequence is verified exactly as pv_verify would verify it alone
 * (same rule, its own prefix_len guard, pending token, K/V pages and in-step rollback); on return
 * accepted_len[i] / next_token[i] hold its results.  The stacked activations use the workspace of
 * caches[0], whose pv_debug_logits then returns all rows in order.  Nothing is changed if a check fails.
 * PV_ENOMEM: the batch needs more attention row groups than the workspace holds (each sequence rounds
 * its gamma x (q heads per kv head) query rows up to a multiple of 32).  Synchronises hip_stream.
 */
int pv_verify_batch(pv_cache *const *caches, int32_t n_seq, const int32_t *prefix_len, const int32_t *draft,
                    const int32_t *gamma, int32_t *accepted_len, int32_t *next_token, void *hip_stream);

/*
 * Verify a draft TREE instead of a draft chain (Sec. 2.2: tree-structured verification explores several
 * candidate continuations in one step; the paper names it as orthogonal to, and combinable with, its
 * pipeline).  tokens[0..n) / parent[0..n) (host arrays): node i carries draft token tokens[i] and hangs
 * under node parent[i] < i, or under the committed prefix if parent[i] = -1; n <= 64.  One block forward
 * in which every node attends to the prefix, its ancestors and itself, at rotary position
 * prefix_len + depth.  Then the stage's own greedy path is followed: starting with expected = pending
 * (unknown: the first root is trusted), the lowest-numbered child of the current node whose token equals
 * `expected` is accepted, and `expected` becomes the stage's prediction after that child; the walk stops
 * where no child matches.  *accepted_len = nodes on the path, *next_token = the prediction after the
 * last of them (pending if none), path[0..accepted_len) (nullable) = their node numbers.  The cache then
 * holds prefix ++ the path's tokens (their K/V moved to consecutive positions), pending = next_token:
 * exactly the state pv_verify reaches when handed the path as a chain.  bf16 models on the matrix path.
 * pv_cache_readmit is not available after this call.  Synchronises hip_stream.
 */
int pv_verify_tree(pv_cache *c, int32_t prefix_len, const int32_t *tokens, const int32_t *parent, int32_t n,
                   int32_t *accepted_len, int32_t *next_token, int32_t *path, void *hip_stream);

/*
 * pv_verify_async for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same step, same results through pv_verify_wait, but it
 * calls no allocating routine (no graph is instantiated, no stream or event is created) and the
 * per-step buffers (activations, operands, partial sums, logits) are taken from one fixed device
 * array inside the library of PV_STATIC_SCRATCH_BYTES bytes, which each GPU the library runs on
 * holds until the process ends, instead of from the cache's workspace; cache state, page table and
 * K/V pages stay in the caller's buffers.  A step that needs more (large vocabulary x gamma, very
 * long max_tokens) is refused with PV_ENOMEM and nothing is changed.  The array is cleared by a
 * kernel at the start of every call.  Every cache of every model on a GPU shares that GPU's array:
 * two such calls that overlap in time on one GPU (different streams or threads) race; calls on
 * one stream, or separated by pv_verify_wait, do not.  The block's logits are not kept for
 * pv_debug_logits.  Instrumentation (pv_profile_select) must be off.
 */
#define PV_STATIC_SCRATCH_BYTES (32u << 20)
int pv_verify_async_static(pv_cache *c, int32_t prefix_len, const int32_t *draft, int32_t gamma, void *hip_stream);

/*
 * Truncate the cache to its first new_len tokens (0 <= new_len <= length, else PV_ERANGE)
 * and forget pending, so the next block's first token is trusted: it is the correction
 * token of the stage that asked for the rollback.  Metadata only.  Synchronises hip_stream.
 */
int pv_rollback(pv_cache *c, int32_t new_len, void *hip_stream);

/*
 * Re-admit positions of the block the last pv_verify / pv_prefill call ran over: set the length
 * to new_len, where (length after that call) <= new_len <= (prefix_len + gamma of that call), and
 * pending to `pending` (-1 = unknown).  Metadata only: the K/V of those positions were written
 * by that call and are still in place.  This exists for drivers that decide acceptance
 * outside the library - the three-stage pipeline benchmark on independent random models draws
 * synthetic acceptances while every stage still runs its real forward pass.  PV_ESTATE if no
 * such block is on record (a rollback, export or set_page_table forgets it), PV_ERANGE if
 * new_len is outside the range above.  Synchronises hip_stream.
 */
int pv_cache_readmit(pv_cache *c, int32_t new_len, int32_t pending, void *hip_stream);

/* ---- state and parity hooks ---- */

int pv_cache_len(const pv_cache *c, int32_t *len, int32_t *pending /* -1 = unknown */);
int pv_cache_set_pending(pv_cache *c, int32_t token_or_minus1, void *hip_stream);

/* Logits of the last verify / last prefill chunk: host_out[rows][vocab] floats, rows = that
 * block's row count (returned in *rows if non-null).  host_out may be NULL to query rows. */
int pv_debug_logits(pv_cache *c, float *host_out, int32_t *rows, void *hip_stream);
/* pred[0..rows) of the last block. */
int pv_debug_pred(pv_cache *c, int32_t *host_out, int32_t *rows, void *hip_stream);
/* Logical K/V of the committed tokens, storage type of the model, laid out
 * [n_layers][2 (K,V)][length][n_kv_heads*head_dim]; nbytes must be at least that size. */
int pv_cache_export(pv_cache *c, void *host_out, size_t nbytes, void *hip_stream);

/* Algorithmic HBM bytes of one step of `gamma` rows at the current length: every streamed
 * weight once + K/V of length+gamma positions once + the K/V written. */
int pv_step_bytes(const pv_cache *c, int32_t gamma, uint64_t *bytes);

/* A step's launch sequence depends only on (row count, mode); by default it is recorded once per
 * such pair as a HIP graph (stream capture on a private stream, thread-local mode) and replayed
 * on the caller's stream afterwards.  enable = 0 switches to plain launches, for comparison and
 * for callers that capture the step into a graph of their own.  Results are identical. */
int pv_cache_use_graphs(pv_cache *c, int32_t enable);

/* ---- instrumentation ---- */

typedef enum {
    PV_PROF_NONE = 0, PV_PROF_QKV = 1, PV_PROF_ATTENTION = 2, PV_PROF_OPROJ = 3, PV_PROF_GATEUP = 4,
    PV_PROF_DOWN = 5, PV_PROF_LMHEAD = 6
} pv_prof_kernel;

/* Select one kernel of the step to be bracketed by HIP events on the step's own stream (every
 * layer's launch of it, every following step) or switch that off.  Resets the counters. */
int pv_profile_select(pv_cache *c, int32_t which);
/* Sum of the bracketed durations (ms), number of launches, and the algorithmic bytes one launch
 * streams (its weights; for attention the K/V of the current length).  Only between steps. */
int pv_profile_read(pv_cache *c, double *total_ms, int64_t *launches, uint64_t *bytes_per_launch);

/* Plain device-to-device copy kernel (k_calib_copy) of `nbytes` bytes, a multiple of 16, both
 * pointers device memory aligned to 16 bytes and not overlapping.  It reads nbytes and writes
 * nbytes of HBM and nothing else: the known quantity against which hardware traffic counters
 * read under a profiler are scaled.  Asynchronous on `hip_stream`. */
int pv_calib_copy(void *d_dst, const void *d_src, size_t nbytes, void *hip_stream);

/* Plain read-only stream (k_calib_read) over `nbytes` bytes of device memory, a multiple of 16,
 * d_src aligned to 16 bytes: every wavefront reads a contiguous slice with 16-byte loads, eight in
 * flight per lane, and nothing is written (d_sink, 16 bytes of device memory, receives a value
 * only if the data happens to XOR to one particular pattern).  It reads nbytes of HBM and nothing
 * else: timed by the caller, it gives the read-stream rate this device reaches on a region of that
 * size, the practical ceiling the weight-streaming kernels are compared with.  Asynchronous on
 * `hip_stream`. */
int pv_calib_read(const void *d_src, size_t nbytes, void *d_sink, void *hip_stream);

const char *pv_strerror(int status);
const char *pv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PIPEVERIFY_H */
