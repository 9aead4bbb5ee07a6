/*
 * treekv.h - C ABI of the TreeKV hot path for AMD MI355X (gfx950).
 *
 * One context holds the state of ONE attention layer: for every (batch element,
 * KV head) an independent fixed-budget KV cache with per-slot importance
 * scores, managed by the paper's Algorithm 1 ("Compression by TreeKV",
 * Section 4.1).  A call attends the new query/queries over the cache
 * (Section 3.1: a = SoftMax(q K^T / sqrt(d)), o = a V), adds the attention
 * probabilities to the slots' scores (Algorithm 1's C and S updates), evicts by the
 * tree rule (its eviction block) and reuses the freed slots for the next tokens.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer owned by the caller; the library
 *     never allocates or frees device memory.  Its own state lives in a
 *     workspace the caller allocates and binds (treekv_workspace_bytes,
 *     treekv_bind_workspace).  treekv_export_state / treekv_import_state take and
 *     restore snapshots of it in a layout-independent form.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls only enqueue work; outputs are valid once the stream has been
 *     synchronised.  Calls on one context must be ordered (one stream, or
 *     events); calls on different contexts are independent.
 *   - Tensors are contiguous, row-major, innermost dimension last.
 *     B = batch, H = query heads, Hkv = KV heads, G = H / Hkv, d = head_dim,
 *     c = budget.  Query head h reads KV head h / G.
 *   - Positions are 0-based indices into the token stream of one sequence.
 *   - Every function returning int returns TREEKV_OK (0) or a negative
 *     treekv_status.  Argument errors are detected before any work is enqueued
 *     and leave the context unchanged.
 *   - Host-side mutable state: none.  Lengths, the eviction index and the free
 *     slot live in the workspace, so identical calls can be captured in a HIP
 *     graph and replayed.
 */
#ifndef TREEKV_H
#define TREEKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum treekv_status {
  TREEKV_OK = 0,
  TREEKV_EINVAL = -1,       /* null pointer, bad size, inconsistent configuration */
  TREEKV_ENOWS = -2,        /* workspace not bound, misaligned or too small        */
  TREEKV_EHIP = -3,         /* a HIP call or kernel launch failed                  */
  TREEKV_EUNSUPPORTED = -4, /* valid request this build has no kernel for          */
  TREEKV_ESCRATCH = -5      /* treekv_decode_step_static: the context needs more scratch than
                               TREEKV_STATIC_SCRATCH_BYTES                            */
} treekv_status;

enum { TREEKV_BF16 = 0, TREEKV_F32 = 1 };      /* storage type of q, k, v and of the cache */
/* The index update Algorithm 1 prints as its last step, idx = (idx+1) mod c + 1, visits every other scope only
 * and contradicts Section 4.1 (whose example has idx take 1, 2, 3, 4 in turn); this library advances idx by one,
 * idx = (idx mod m) + 1, and has no flag for the printed form. */
enum {
  TREEKV_KEEP_LEFT = 1,          /* flags: ablation of Section 5.4 (always keep the left slot of the scope,
                                    ignore the scores)                                                   */
  TREEKV_SCORE_ACCUMULATED = 4,  /* importance = accumulated weight S instead of the average S / C
                                    (Section 4.1, "Importance Score": the criterion tried next to the
                                    average); Algorithm 1's averaging step is skipped, the scope compares S     */
  TREEKV_POSITION_RERANK = 8     /* positions re-assigned after eviction (Section 4.1, "Position Encoding"):
                                    q and k are given WITHOUT positional encoding and the cache keeps them so;
                                    at every decode step the cached tokens and the new one, in position order,
                                    take the positions 0 .. n-1 (the paper's example: {0,1,2,3,7,8,9} and token
                                    10 get 0..7) and the rotary encoding of those positions is applied to the
                                    keys and the query inside the step.  Rotary encoding as defined by its
                                    authors: dimensions (2i, 2i+1) form a plane turned by
                                    position * rope_base^(-2i/d); a model that pairs (i, i + d/2) permutes the
                                    head dimension of q and k accordingly.  treekv_prefill_chunk scores a chunk
                                    before anything of it is evicted: the n cached tokens are at positions
                                    0 .. n-1 and chunk token i (and its query) at n + i -- for a one-token chunk
                                    the decode step's rule.  treekv_prefill_prompt takes its queries and keys
                                    unencoded too: nothing has been evicted when the window scores the prompt,
                                    so key j is at position j and window query i at len - block + i.  The cache
                                    always holds the keys unencoded.                                          */
};

enum { TREEKV_DEFAULT_LAYOUT = -1 };           /* n_sink = n_recent = this: 4 sinks, budget/2 tree slots, the rest recent */

typedef struct treekv_ctx treekv_ctx;          /* opaque, host memory, owns no device memory */

typedef struct treekv_config {
  int32_t budget;        /* c: slots kept after every call (Algorithm 1, input "cache size c") */
  int32_t q_heads;       /* H                                                                  */
  int32_t kv_heads;      /* Hkv, must divide H; the scores of a KV head add up the attention
                            probabilities of its G query heads                               */
  int32_t head_dim;      /* d: 64 or 128                                                       */
  int32_t batch;         /* B independent sequences, all advancing together                   */
  int32_t dtype;         /* TREEKV_BF16 or TREEKV_F32                                          */
  int32_t n_sink;        /* leading tokens never evicted  (Section 5.2: 4)                     */
  int32_t n_recent;      /* trailing tokens never evicted (Section 5.2: 508 of 1024); both
                            TREEKV_DEFAULT_LAYOUT: the layout treekv_init chooses             */
  float softmax_scale;   /* multiplies q.k; 0 selects 1/sqrt(head_dim) (Section 3.1)           */
  int32_t flags;         /* 0, or an OR of TREEKV_KEEP_LEFT, TREEKV_SCORE_ACCUMULATED,
                            TREEKV_POSITION_RERANK                                             */
  int32_t max_chunk;     /* largest `len` treekv_prefill_chunk will be given; 0 selects 512    */
  int32_t kv_splits;     /* decode: workgroups per (batch, KV head); 0 lets the library choose */
  int32_t max_prompt;    /* longest `len` treekv_prefill_prompt will be given; 0: that call is not used
                            (its scratch, 4 bytes per token and (batch, KV head), is then left out)    */
  float rope_base;       /* TREEKV_POSITION_RERANK: base of the rotary angles; 0 selects 10000            */
} treekv_config;

/*
 * treekv_init - the three-argument form of the problem statement: one sequence
 * (B = 1), Hkv = H = heads, bf16, scale 1/sqrt(head_dim), and the cache layout
 * of Section 5.2 scaled to the budget: 4 sink tokens, budget/2 tree slots, the
 * rest recent tokens (4 + 512 + 508 at budget 1024).  Needs budget >= 16.
 * Allocates only host memory.  *out is set on success.
 */
int treekv_init(treekv_ctx** out, int budget, int heads, int head_dim);

/* treekv_init_ex - full configuration.  Requires budget - n_sink - n_recent >= 1 (or both TREEKV_DEFAULT_LAYOUT
 * and budget >= 16). */
int treekv_init_ex(treekv_ctx** out, const treekv_config* cfg);

/* Frees the host-side context (not the workspace, which is the caller's). */
void treekv_destroy(treekv_ctx* ctx);

/* The effective configuration (defaults filled in). */
int treekv_get_config(const treekv_ctx* ctx, treekv_config* out);

/* Bytes of device memory the context needs (cache rows, scores, positions, order
 * arrays, split-KV and prefill scratch).  0 for a null context. */
size_t treekv_workspace_bytes(const treekv_ctx* ctx);

/* Binds caller-allocated device memory (256-byte aligned, at least
 * treekv_workspace_bytes).  Does not touch the memory; call treekv_reset next. */
int treekv_bind_workspace(treekv_ctx* ctx, void* dev_ptr, size_t bytes);

/* Algorithm 1, initialisation: empty cache, idx at the first scope, position counter 0. */
int treekv_reset(treekv_ctx* ctx, void* stream);

/*
 * treekv_decode_step - one iteration of Algorithm 1's loop (append to index advance) for every
 * (batch, KV head), without the projections that open the loop.
 *   q [B, H, d], k [B, Hkv, d], v [B, Hkv, d]   storage dtype, read only
 *   out        [B, H, d] float32: o = SoftMax(q K^T * scale) V over the cache
 *              including the new token, computed before the eviction
 *   retained   [B, Hkv, c] int32: positions kept after the step, ascending,
 *              padded with -1 while the cache is still filling
 *   n_retained [B, Hkv] int32 (may be NULL)
 *   evicted    [B, Hkv] int32 (may be NULL): position evicted at this step, or -1
 */
int treekv_decode_step(treekv_ctx* ctx, const void* q, const void* k, const void* v, void* out,
                       int32_t* retained, int32_t* n_retained, int32_t* evicted, void* stream);

/*
 * treekv_decode_step_static - treekv_decode_step with the same arguments, results and kernels, for callers that can
 * neither allocate device memory nor hand the library scratch of their own for this: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  The only scratch a decode step uses -- the scaled logits
 * [U][G][c+1] float32 and the per-slice partial results [U][kv_splits][G][d+2] float32 that the two-kernel shape
 * (kv_splits > 1) passes from its first kernel to its second -- lives in a fixed array of
 * TREEKV_STATIC_SCRATCH_BYTES inside the library's device image instead of the bound workspace (the one-kernel
 * shape, kv_splits = 1, uses none).  Each GPU holds one such array until the process ends; every call on a GPU,
 * from any context, shares it: calls that may overlap on one GPU (different streams without ordering) race and
 * must not both use this entry point.  Nothing in the array has to survive from one call to the next and nothing
 * has to start at zero (the first kernel writes every word the second reads).  No hipMalloc, hipFree or other
 * allocating call is made; the array's address is looked up once per device, on the first call there.
 * Errors: as treekv_decode_step, and TREEKV_ESCRATCH (nothing enqueued) if the context's logits and partials
 * exceed TREEKV_STATIC_SCRATCH_BYTES.
 */
enum { TREEKV_STATIC_SCRATCH_BYTES = 16 << 20 };
int treekv_decode_step_static(treekv_ctx* ctx, const void* q, const void* k, const void* v, void* out,
                              int32_t* retained, int32_t* n_retained, int32_t* evicted, void* stream);

/*
 * treekv_prefill_chunk - `len` consecutive tokens at once (1 <= len <= max_chunk).
 * Row i attends the cache as it was before the call plus the chunk's tokens
 * 0..i (causal inside the chunk).  All rows' probabilities are added to the
 * scores and counts; the averaged scores are then frozen and Algorithm 1's
 * append / compare / evict / advance is replayed for the
 * chunk's tokens in order.  len = 1 is exactly treekv_decode_step.
 *   Q [B, len, H, d], K [B, len, Hkv, d], V [B, len, Hkv, d]   storage dtype
 *   out        [B, len, H, d] float32
 *   retained   [B, Hkv, c] int32, n_retained [B, Hkv] (may be NULL): as above
 *   evicted    [B, Hkv, len] int32 (may be NULL): position evicted when the
 *              chunk's i-th token was appended, or -1
 * With bf16 storage the two contractions run on the matrix pipe; with fp32 storage
 * they run, row by row, on the vector ALUs (held to 1e-5, not a fast path), for at most
 * 10240 visible columns (budget + 1 + len; TREEKV_EUNSUPPORTED beyond).
 */
int treekv_prefill_chunk(treekv_ctx* ctx, const void* Q, const void* K, const void* V, int len,
                         void* out, int32_t* retained, int32_t* n_retained, int32_t* evicted,
                         void* stream);

/*
 * treekv_prefill_prompt - the paper's own prefilling stage (Section 4.2): a whole prompt of `len` tokens is
 * compressed in one shot, block by block.  The prompt is cut into blocks of `block` tokens; the queries of
 * its last block (the observation window) attend the entire prompt causally; a token's importance is its
 * attention weight averaged over the window queries that see it (S / C of Algorithm 1,
 * for those queries; the G query heads of a KV head add up); a block's importance is the mean over its
 * tokens; Algorithm 1's append / compare / evict / advance then runs with blocks in the
 * place of tokens and these scores frozen: budget / block blocks are kept, ceil(n_sink / block) leading
 * and ceil(n_recent / block) trailing blocks are never evicted.  The call REPLACES the context's state
 * (the context must have been reset once since its workspace was bound).  Afterwards the cache holds
 * the kept blocks' tokens and decoding can go on: the paper does not say how; here a kept token's
 * averaged score stays its window average (its count becomes len - position, its accumulated weight
 * that count times the average) and token-level eviction starts at the first scope.
 *   Qw [B, block, H, d]: queries of the prompt's last `block` tokens; K, V [B, len, Hkv, d]: the whole
 *   prompt; storage dtype, read only
 *   retained   [B, Hkv, c] int32: positions kept, ascending, padded with -1 (len < c keeps everything)
 *   n_retained [B, Hkv] int32 (may be NULL)
 *   evicted_blocks [B, Hkv, len / block] int32 (may be NULL): the block evicted when block i was
 *              appended, or -1
 *   token_scores [B, Hkv, len] float32 (may be NULL): the tokens' averaged window attention
 * With fp32 storage the window's scores are computed on the vector ALUs, one window query at a time (not a
 * fast path), for len <= 32768.
 * Errors: TREEKV_EINVAL unless 1 <= block <= len <= max_prompt, block divides len and budget, and
 * budget / block - ceil(n_sink / block) - ceil(n_recent / block) >= 1; TREEKV_EUNSUPPORTED if
 * block * G > 128, or with fp32 storage as said above.
 */
int treekv_prefill_prompt(treekv_ctx* ctx, const void* Qw, const void* K, const void* V, int len, int block,
                          int32_t* retained, int32_t* n_retained, int32_t* evicted_blocks,
                          float* token_scores, void* stream);

/*
 * treekv_scores - accumulated attention weights S (Algorithm 1's score update) of the
 * retained tokens, in the order of `retained`; the count C is
 * t - position + 1 with t the last processed position, so Sbar = S / C.
 *   scores [B, Hkv, c] float32, padded with 0.
 */
int treekv_scores(treekv_ctx* ctx, float* scores, void* stream);

/*
 * treekv_gather_kv - the retained keys and values in the order of `retained`
 * (the compacted cache), for callers that want it contiguous.
 *   K_out, V_out [B, Hkv, c, d] storage dtype; rows past n_retained are zeroed.
 */
int treekv_gather_kv(treekv_ctx* ctx, void* K_out, void* V_out, void* stream);

/*
 * treekv_wavelet_components - the analysis the method is motivated by (Sections 3.2-3.3), stateless.  For each
 * of `heads` heads at one generation step the signal is s[n] = a[n] * v[n] (the information position n
 * contributes to the attention output, Section 3.3); every column of s is decomposed along the sequence by
 * `levels` levels of the Haar filter pair (Section 3.2) and Rec(D_l), the part of the signal carried by the
 * level-l detail coefficients alone, is rebuilt; the result is its magnitude per position.
 *   a [heads, t] float32: attention weights;  V [heads, t, d] of storage type `dtype`;  read only
 *   per_head [heads, levels, t] float32: |Rec(D_l)[n]| averaged over the d columns (l = 1 first, the highest
 *              frequency)
 *   mean     [levels, t] float32 (may be NULL): per_head averaged over the heads (added in an order that
 *              depends on the number of heads only: results repeat bit for bit)
 * Positions pair up as (1,2), (3,4), .. counted from 1, as in the printed reconstruction formula.
 * Errors: TREEKV_EINVAL for null pointers, sizes below 1 or a length 2^levels does not divide;
 * TREEKV_EUNSUPPORTED for levels > 5, d other than 64 or 128, heads > 65535.
 */
int treekv_wavelet_components(const float* a, const void* V, int dtype, int heads, int t, int d, int levels,
                              float* per_head, float* mean, void* stream);

/*
 * Snapshots: Algorithm 1's state (S, C, K, V, idx; C is t - position) of every (batch, KV head) unit,
 * in position order, independent of how the workspace lays the cache out.  A snapshot is one device buffer of
 * treekv_state_bytes(ctx) bytes, 256-byte aligned, holding six arrays at the byte offsets treekv_get_state_layout
 * reports (U = B * Hkv units, c = budget):
 *   header    [U][4] int32   n (tokens kept), t (tokens processed so far), idx (the paper's, 1 .. m), 0
 *   positions [U][c] int32   stream positions of the kept tokens, ascending; -1 past n
 *   slots     [U][c] int32   the cache row each token sits in (0 .. c); -1 past n.  Restoring rows to the same
 *                            slots makes the steps after an import repeat bit for bit what followed the export.
 *                            A snapshot built by hand may set slots[u][0] = -1: token i then takes row i.
 *   S         [U][c] float32 accumulated attention weight of each kept token (Algorithm 1's S); 0 past n
 *   K, V      [U][c][d]      storage dtype; the kept tokens' rows, zero past n
 */
typedef struct treekv_state_layout {
  size_t header, positions, slots, S, K, V;   /* byte offsets into the snapshot */
  size_t bytes;                               /* its total size                  */
} treekv_state_layout;

size_t treekv_state_bytes(const treekv_ctx* ctx);                      /* 0 for a null context */
int treekv_get_state_layout(const treekv_ctx* ctx, treekv_state_layout* out);

/* treekv_export_state - writes a snapshot of the context, as it is once the calls enqueued before on `stream`
 * have run, to dst (device memory, caller-owned).  TREEKV_EINVAL if dst is null, misaligned or `bytes` too small. */
int treekv_export_state(treekv_ctx* ctx, void* dst, size_t bytes, void* stream);

/*
 * treekv_import_state - replaces the context's state by a snapshot (of a context with the same configuration;
 * it may come from treekv_export_state or be built by the caller, e.g. from another implementation's state).
 * The context must have been reset once since its workspace was bound.  Every unit's snapshot is checked on the
 * device: 0 <= n <= c, 1 <= idx <= m; while the cache fills (n < c) nothing has been evicted: t = n, idx = 1,
 * positions 0 .. n-1; once it is full: t >= n, positions ascending and below t, the first n_sink of them
 * 0 .. n_sink-1, the last n_recent of them t-n_recent .. t-1, and slots either unset or all different.
 *   status [U] int32 (device, may be NULL): TREEKV_OK or TREEKV_EINVAL per unit.  A unit that fails the check
 *   is left EMPTY (as after treekv_reset); the others are imported.
 * TREEKV_EINVAL (nothing enqueued) if src is null, misaligned or `bytes` too small.
 */
int treekv_import_state(treekv_ctx* ctx, const void* src, size_t bytes, int32_t* status, void* stream);

/* Static description of a status code. */
const char* treekv_strerror(int status);

/* Text of the HIP error behind the last TREEKV_EHIP this context returned ("" if none).  An error that an
 * unrelated, earlier HIP call of the calling thread left pending is dropped when an entry point starts, not
 * reported as this library's. */
const char* treekv_last_hip_error(const treekv_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* TREEKV_H */
