/*
 * wgkv.h -- C ABI of the Write-Gated KV hot path for AMD MI355X (gfx950).
 *
 * What the library does ("KV Admission: Learning What to Write for Efficient
 * Long-Context LLM Inference"):
 *   - a per-token, per-KV-head write gate decides admission before any write:
 *     admit <=> g >= tau (Sec. 3.3, last sentence);
 *   - every head keeps a dual cache: a ring-buffer local window of W_local slots
 *     and a growing global cache, both mapped through per-head page tables onto
 *     one physical pool of fixed-size pages (Sec. 4.1);
 *   - prefill writes the final W_local tokens to the local cache and earlier
 *     tokens to the global cache only if admitted (Sec. 4.2, "Initial cache
 *     population"); decode promotes lazily: the token leaving the window is
 *     inspected and, if its stored score passes tau, moved to the global cache
 *     before the new token takes its slot (Sec. 4.3, steps (1)-(3));
 *   - attention reads local window + global cache of the query's KV head,
 *     ragged across heads (Sec. 4.3 last sentence; App. A; App. E "Decode
 *     phase": split the ragged work into uniform pieces, then reduce), which is
 *     attention under the vertical-slash mask of Sec. 4.2.
 *
 * Conventions
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are host
 *     addresses.  The library never allocates, frees or owns device memory: the
 *     caller provides the pool, the metadata block and a workspace and keeps
 *     them alive until wgkv_destroy.  The handle itself is host heap memory.
 *   - All path calls (prefill_admit, decode_step, attend, gate_scores, free_seq)
 *     only enqueue kernels on the given stream (a hipStream_t passed as void*)
 *     and return; calls on one pool must be issued in stream order.  Small host
 *     arrays are read before the call returns.  Only wgkv_status and
 *     wgkv_tune_decode_attention synchronise.
 *   - Return value: 0 = WGKV_OK, negative = error.  Argument errors and page
 *     exhaustion are detected on the host before anything is enqueued and leave
 *     all state untouched.
 *   - Positions are 0-based; a (sequence, layer) that has seen t tokens holds
 *     positions [max(0,t-W), t) in its ring (position p in slot p mod W) and the
 *     admitted positions below t-W, ascending, in its global cache.
 *   - Page allocation order (the paper fixes none; this rule makes page tables
 *     reproducible): free_stack[i] = n_pages-1-i at init, pop takes
 *     free_stack[--free_top]; within a call, demands are served unit by unit in
 *     (position of the sequence in the call, kv head) order, a unit's
 *     ceil(W/P) local pages (taken at its first use) before its global pages.
 */
#ifndef WGKV_H
#define WGKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct wgkv_pool wgkv_pool; /* opaque host-side handle */
typedef void *wgkv_stream;          /* hipStream_t */

enum { WGKV_F32 = 0, WGKV_BF16 = 1 };

enum {
    WGKV_OK = 0,
    WGKV_ERR_INVALID_ARG = -1,
    WGKV_ERR_OUT_OF_PAGES = -2, /* host-side bound on free pages would go negative */
    WGKV_ERR_PT_OVERFLOW = -3,  /* a page-table row could exceed max_global_pages_per_head */
    WGKV_ERR_HIP = -4,          /* a HIP runtime call failed */
    WGKV_ERR_DEVICE_FLAG = -5,  /* the device-side sticky error flag is set */
    WGKV_ERR_WORKSPACE = -6,    /* workspace too small for this call */
    WGKV_ERR_HOST_MEMORY = -7,  /* the host handle could not be allocated */
    WGKV_ERR_ADMIT_BOUND = -8,  /* device flag only: a unit admitted more tokens than the caller's bound */
    WGKV_ERR_NOT_PROMOTED = -9  /* device flag only: a decode step that relied on wgkv_decode_promote found a
                                   head whose promotion had not been done ahead */
};

#define WGKV_MAX_CALL_SEQS 128  /* sequences per call */
#define WGKV_MAX_CALL_UNITS 1024 /* sequences per call x kv heads */

typedef struct {
    int32_t n_layers, n_q_heads, n_kv_heads; /* n_q_heads % n_kv_heads == 0, group size 1,2,4 or 8 */
    int32_t head_dim;                         /* 64 or 128 */
    int32_t dtype;                            /* element type of K, V, Q and the pool */
    int32_t page_size;                        /* tokens per page P, a power of two (paper: 16) */
    int32_t w_local;                          /* local window W_local >= 1 (paper: 256) */
    int32_t max_seqs;                         /* sequence slots */
    int32_t max_global_pages_per_head;        /* width of a global page-table row */
    int64_t n_pages;                          /* physical pages in the pool, < 2^31 */
} wgkv_config;

/* Byte offsets of the arrays inside the metadata block (S = max_seqs, L =
 * n_layers, H = n_kv_heads, NLP = ceil(W/P), MGP = max_global_pages_per_head):
 *   seq_len    int32 [S][L]          tokens seen
 *   global_len int32 [S][L][H]       global-cache length G_h
 *   local_pt   int32 [S][L][H][NLP]  physical page of each ring page, -1 = none yet
 *   global_pt  int32 [S][L][H][MGP]  physical page of each global page, -1 = unused
 *   ring_g     float [S][L][H][W]    stored score of each ring slot
 *   free_stack int32 [n_pages]       LIFO of free pages
 *   free_top   int32                 number of free pages
 *   err_flag   int32                 sticky: 0 ok, else first WGKV_ERR_* seen on device
 *   ahead      int32 [S][L][H]       (t << 1) | promoted once wgkv_decode_promote has handled the
 *                                    step that feeds token t of this head, else -1
 *   unit_counters int32 [WGKV_MAX_CALL_UNITS]  scratch of wgkv_attend, zero between calls
 * Pool: element [page][0=K,1=V][slot 0..P-1][head_dim]. */
typedef struct {
    size_t seq_len, global_len, local_pt, global_pt, ring_g, free_stack, free_top, err_flag;
    size_t unit_counters;
    size_t ahead;
    size_t total_bytes;
    int32_t n_local_pages;
} wgkv_meta_layout;

/* Sizes of the caller-provided device buffers.  workspace_bytes is enough for
 * any call with at most max_call_seqs sequences and max_call_tokens tokens in
 * total (a decode call has one token per sequence).  Any output may be NULL. */
int wgkv_query_sizes(const wgkv_config *cfg, int32_t max_call_seqs, int64_t max_call_tokens,
                     size_t *pool_bytes, size_t *meta_bytes, size_t *workspace_bytes);

/* Where each metadata array lives (so that a caller can snapshot or inspect state). */
int wgkv_get_meta_layout(const wgkv_config *cfg, wgkv_meta_layout *out);

/* Sec. 4.1.  Validates cfg, adopts pool_dev (>= pool_bytes, 256-byte aligned)
 * and meta_dev (>= meta_bytes), enqueues one kernel that builds the free stack
 * and clears lengths and tables, and returns a handle in *out. */
int wgkv_init_pool(const wgkv_config *cfg, void *pool_dev, size_t pool_bytes, void *meta_dev,
                   size_t meta_bytes, wgkv_stream stream, wgkv_pool **out);

/* Sec. 3.2 gate equation without the hidden layer (the linear write gate of the
 * chunked-prefill workload): g[t][h] = sigmoid(w[h] . hidden[t]).
 *   hidden_dev [n_tokens][hidden_dim], gate_w_dev [n_kv_heads][hidden_dim], both of
 *   `dtype`; g_out_dev float [n_tokens][n_kv_heads]; fp32 accumulation.
 * hidden_dim must be a multiple of 8, n_kv_heads at most 16, both matrices 16-byte aligned
 * (INVALID_ARG otherwise). */
int wgkv_gate_scores(int32_t dtype, int64_t n_tokens, int32_t hidden_dim, int32_t n_kv_heads,
                     const void *hidden_dev, const void *gate_w_dev, float *g_out_dev,
                     wgkv_stream stream);

/* Sec. 3.2, "Write-Gated Attention" in its log-space form (the attention that trains the
 * gate): for every sequence of the call, query position i and query head qh (kv head
 * h = qh / (n_q_heads / n_kv_heads)),
 *   s_ij  = scale * q[i][qh] . k[j][h] + log(max(1(i - j < w_local), g[j][h]) + eps),  j <= i
 *   out[i][qh] = sum_j softmax_j(s_ij) v[j][h],      lse[i][qh] = log sum_j exp(s_ij).
 * The paper says only that eps is small; it is an argument (eps >= 0).
 *   n_tokens_host [n_seqs] : tokens per sequence (host); rows of all tensors are the sequences
 *                            packed one after the other, at most 2^24 - 1 rows in total
 *   q_dev [rows][n_q_heads][head_dim], k_dev, v_dev [rows][n_kv_heads][head_dim] bf16, 16-byte
 *   aligned; g_dev float [rows][n_kv_heads]
 *   out_dev float [rows][n_q_heads][head_dim] (16-byte aligned), lse_dev float [rows][n_q_heads]
 * Products run on the matrix cores in bf16 with fp32 accumulation; the weights are rounded to
 * bf16 before the second product and the denominator sums the rounded weights.
 * Supported: dtype WGKV_BF16, head_dim 128, n_q_heads = 4 * n_kv_heads; anything else returns
 * INVALID_ARG.  All buffers are device memory owned by the caller; the call only enqueues work
 * on `stream`.  Errors: INVALID_ARG, HIP. */
int wgkv_soft_attn_forward(int32_t dtype, int32_t n_seqs, const int32_t *n_tokens_host,
                           int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                           int32_t w_local, const void *q_dev, const void *k_dev,
                           const void *v_dev, const float *g_dev, float scale, float eps,
                           float *out_dev, float *lse_dev, wgkv_stream stream);

/* Bytes of workspace wgkv_soft_attn_backward needs for total_tokens packed rows. */
size_t wgkv_soft_attn_workspace_bytes(int64_t total_tokens, int32_t n_q_heads);

/* Gradients through wgkv_soft_attn_forward (same Sec. 3.2 equations) of a loss with
 * dLoss/dOut = dout.  With p_ij = exp(s_ij - lse_i):
 *   dv[j][h] = sum_{i, qh of h} p_ij dout[i][qh]
 *   dS_ij    = p_ij (dout[i][qh] . v[j][h] - dout[i][qh] . out[i][qh])
 *   dq[i][qh] = scale sum_j dS_ij k[j][h],   dk[j][h] = scale sum_{i, qh of h} dS_ij q[i][qh]
 *   dg[j][h] = sum over (i, qh of h) where g_j exceeds 1(i - j < w_local) of dS_ij / (g_j + eps)
 * Inputs as in the forward call plus its results out_dev and lse_dev, and
 *   dout_dev bf16 [rows][n_q_heads][head_dim], 16-byte aligned.
 * Outputs (all float, 16-byte aligned, fully overwritten): dq_dev [rows][n_q_heads][head_dim],
 * dk_dev, dv_dev [rows][n_kv_heads][head_dim], dg_dev [rows][n_kv_heads].
 * workspace_dev: wgkv_soft_attn_workspace_bytes(rows, n_q_heads) bytes, contents undefined
 * before and after.  p and dS are rounded to bf16 before the products that consume them.
 * Every output element is written by exactly one wave in a fixed order: results do not change
 * from run to run.  Errors: INVALID_ARG, WORKSPACE, HIP. */
int wgkv_soft_attn_backward(int32_t dtype, int32_t n_seqs, const int32_t *n_tokens_host,
                            int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                            int32_t w_local, const void *q_dev, const void *k_dev,
                            const void *v_dev, const float *g_dev, float scale, float eps,
                            const float *out_dev, const float *lse_dev, const void *dout_dev,
                            float *dq_dev, float *dk_dev, float *dv_dev, float *dg_dev,
                            void *workspace_dev, size_t workspace_bytes, wgkv_stream stream);

/* Sec. 3.3, sparsity term of the training objective over n scores out of n_total (the
 * paper's L * H * T; a caller that holds the scores layer by layer adds up the calls):
 *   *loss_dev = sum_x (g[x] + g[x] (1 - g[x])) / n_total,   dg_dev[x] = (2 - 2 g[x]) / n_total.
 *   g_dev float [n]; loss_dev one float; dg_dev float [n] or NULL; workspace_dev at least
 *   WGKV_SPARSITY_WS_BYTES bytes, contents undefined before and after.
 * fp32 sums in a fixed order (the last stage in double): the value repeats bit for bit.
 * Device buffers are the caller's; the call only enqueues work on `stream`.
 * Errors: INVALID_ARG (n < 0, n > n_total, NULL), WORKSPACE, HIP. */
#define WGKV_SPARSITY_WS_BYTES 4096
int wgkv_sparsity_loss(const float *g_dev, int64_t n, int64_t n_total, float *loss_dev, float *dg_dev,
                       void *workspace_dev, size_t workspace_bytes, wgkv_stream stream);

/* Sec. 3.2, feature equation and gate equation (the Write-Gate MLP), per token t and
 * kv head h:  x = [RMSNorm(k[t][h]) ; RMSNorm(k_rope[t][h])],
 *             g[t][h] = sigmoid(W2[h] . GELU(W1[h] x + b1[h]) + b2[h]).
 * The paper leaves width, GELU flavour and RMSNorm constants open: width is an
 * argument, GELU is the exact one (erf), RMSNorm(v) = v / sqrt(mean(v^2) + eps) has no
 * learnable scale.  With bf16 inputs the normalised features are rounded to bf16 before
 * the first product; accumulation, GELU and sigmoid are fp32.
 *   k_dev, k_rope_dev : [n_tokens][n_kv_heads][head_dim] of `dtype` (keys before and
 *                       after the rotary embedding), 16-byte aligned
 *   w1_dev [n_kv_heads][width][2*head_dim], w2_dev [n_kv_heads][width] of `dtype`;
 *   b1_dev float [n_kv_heads][width], b2_dev float [n_kv_heads]
 *   g_out_dev float [n_tokens][n_kv_heads]
 * All buffers are device memory owned by the caller; the call only enqueues work on
 * `stream`.  bf16 with head_dim 64 or 128 and width a multiple of 32 runs on the matrix
 * cores, every other shape on a plain kernel.  Errors: INVALID_ARG, HIP. */
int wgkv_gate_mlp_scores(int32_t dtype, int64_t n_tokens, int32_t n_kv_heads, int32_t head_dim,
                         int32_t width, const void *k_dev, const void *k_rope_dev,
                         const void *w1_dev, const float *b1_dev, const void *w2_dev,
                         const float *b2_dev, float eps, float *g_out_dev, wgkv_stream stream);

/* Sec. 4.2 "Initial cache population", also for one chunk of a chunked prefill:
 * feeds n_tokens_host[b] new tokens of layer `layer` to sequence seq_ids_host[b]
 * (distinct ids, n_seqs <= WGKV_MAX_CALL_SEQS).  Tokens that leave the window in
 * this call (from the old ring or from the chunk) are appended to the global
 * cache in position order iff their score >= tau, with new pages popped as
 * needed; the last min(W, t) tokens end up in the ring with their scores.
 *   k_dev, v_dev : [sum T][n_kv_heads][head_dim] of cfg.dtype, sequences packed
 *   g_dev        : float [sum T][n_kv_heads] scores, or NULL to compute them from
 *                  hidden_dev [sum T][hidden_dim] and gate_w_dev (see wgkv_gate_scores)
 *   admit_mask_out_dev : optional uint8 [sum T][n_kv_heads], 1(g >= tau)
 * The gate form (g_dev == NULL) has the limits of wgkv_gate_scores: at most 16 kv heads,
 * hidden_dim a multiple of 8, hidden_dev and gate_w_dev 16-byte aligned.
 * Errors: INVALID_ARG, OUT_OF_PAGES / PT_OVERFLOW (from host-side worst-case
 * bounds: every leaving token counted as admitted; wgkv_status tightens them),
 * WORKSPACE, HIP. */
int wgkv_prefill_admit(wgkv_pool *pool, int32_t layer, int32_t n_seqs,
                       const int32_t *seq_ids_host, const int32_t *n_tokens_host,
                       const void *k_dev, const void *v_dev, const float *g_dev,
                       const void *hidden_dev, const void *gate_w_dev, int32_t hidden_dim,
                       float tau, uint8_t *admit_mask_out_dev, void *workspace_dev,
                       size_t workspace_bytes, wgkv_stream stream);

/* The same call for a pool sized for the admitted cache rather than for the worst case
 * (Sec. 4.2 "Initial cache population"; Sec. 3.3: the gate admits a small share of the tokens).
 * max_admitted_per_head >= 0 is the caller's promise that no (sequence, kv head) of this call
 * admits more than that many tokens to its global cache in this call.  The host-side page
 * bounds then count min(leaving tokens, max_admitted_per_head) per head instead of all leaving
 * tokens, so a loop of chunks needs no wgkv_status (a device synchronisation) between calls
 * to stay inside a pool of that size.  The device checks the promise before it changes
 * anything: when a head admits more, the call leaves the pool exactly as it was and sets the
 * sticky device flag to WGKV_ERR_ADMIT_BOUND (seen by the next wgkv_status, which also
 * re-reads the token counts; the host's counts of that call are then ahead of the device's
 * until it does).  Everything else as wgkv_prefill_admit.
 * Errors: those of wgkv_prefill_admit; INVALID_ARG for a negative bound. */
int wgkv_prefill_admit_bounded(wgkv_pool *pool, int32_t layer, int32_t n_seqs,
                               const int32_t *seq_ids_host, const int32_t *n_tokens_host,
                               const void *k_dev, const void *v_dev, const float *g_dev,
                               const void *hidden_dev, const void *gate_w_dev, int32_t hidden_dim,
                               float tau, int32_t max_admitted_per_head, uint8_t *admit_mask_out_dev,
                               void *workspace_dev, size_t workspace_bytes, wgkv_stream stream);

/* Sec. 4.3 lazy promotion, one new token per sequence: the victim in slot
 * t mod W (if t >= W) is appended to the global cache iff its stored score
 * >= tau, then (k_new, v_new, g_new) take the slot and t advances.
 *   k_new_dev, v_new_dev : [n_seqs][n_kv_heads][head_dim];  g_new_dev : float [n_seqs][n_kv_heads]
 *   promoted_out_dev     : optional uint8 [n_seqs][n_kv_heads]
 * HIP graphs: this call and the decode form of wgkv_attend enqueue kernels only (no
 * synchronisation, no memset, no allocation) and the kernels take the token counts from
 * device memory, so a captured sequence of them can be replayed: every replay is one more
 * token, read from whatever the input buffers hold at that time.  Capturing runs nothing on
 * the device, and the host-side bookkeeping sees neither captures correctly nor replays at
 * all: call wgkv_status after the last replay and before the next direct call.  While
 * replaying, a step that finds no free page (or a full page table) sets the device error
 * flag and changes nothing.
 * Errors: INVALID_ARG, OUT_OF_PAGES / PT_OVERFLOW (host-side bounds), HIP. */
int wgkv_decode_step(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                     const void *k_new_dev, const void *v_new_dev, const float *g_new_dev,
                     float tau, uint8_t *promoted_out_dev, wgkv_stream stream);

/* Sec. 4.3 steps (1)-(2) of ALL layers ahead of time.  Whether the victim of the coming token
 * is promoted depends on the score stored with it and on the token count only, not on the
 * layer's new key and value: this call does the victim test, the page hand-out and the row move
 * of every layer of the named sequences in two launches, and the wgkv_decode_step calls of the
 * same token (one per layer, as before, same tau) then only write the ring, which takes a layer's
 * step off the path between its projections and its attention.  Optional: without it
 * wgkv_decode_step does all three steps itself.  The promotion masks and the cached rows are
 * the same either way, and so are the page tables bit for bit (pages are taken in the order
 * layer, sequence of the call, head, as the layers' own steps take them) when the steps name
 * the same sequences in the same order as this call and none of them receives its very first
 * token in this step (its ring pages are handed out by its decode steps, after the global
 * pages of all layers instead of in between); otherwise the same pages end up under other
 * numbers.
 * Every layer of a sequence must hold the same number of tokens (INVALID_ARG otherwise).
 * After this call the next call on those sequences must be wgkv_decode_step for each layer:
 * wgkv_prefill_admit on a layer promoted ahead is refused (INVALID_ARG).  Calling it twice
 * for the same token changes nothing the second time.
 * HIP graphs: capture it together with the layers' steps.  A replayed wgkv_decode_step whose
 * promotion is not in the graph finds no promotion done, changes nothing and sets the device
 * flag to WGKV_ERR_NOT_PROMOTED.  Running out of pages sets the flag like a replayed step does
 * (all layers or none).
 * Errors: INVALID_ARG, OUT_OF_PAGES / PT_OVERFLOW (host-side bounds), HIP. */
int wgkv_decode_promote(wgkv_pool *pool, int32_t n_seqs, const int32_t *seq_ids_host, float tau,
                        wgkv_stream stream);

/* Attention of the queries of layer `layer` over what the cache holds.
 * Decode (every n_q_host[b] == 1, k_chunk_dev == NULL): call after
 * wgkv_decode_step; query head hq reads the valid ring slots and the global
 * cache of kv head hq / (n_q_heads / n_kv_heads) (Sec. 4.3; Sec. 2.1 equation).
 * Prefill chunk (k_chunk_dev, v_chunk_dev, g_chunk_dev given; n_q_host[b] = chunk
 * length T_b): call BEFORE wgkv_prefill_admit of the same chunk; query i of the
 * chunk (position t+i) sees the global cache, ring positions j with
 * (pos_i - j < W or stored g_j >= tau) and chunk keys j <= i with
 * (i - j < W or g_j >= tau)  (Sec. 4.2 mask equation).
 * With dtype bf16, head_dim 128 and 4 query heads per kv head (the paper's models) the
 * prefill-chunk form runs on the matrix cores; every other shape the pool accepts takes a plain
 * kernel (fp32 accumulation, one wave per query and head: correct, not fast).  k_chunk_dev and
 * v_chunk_dev must be 16-byte aligned.
 *   q_dev   : [sum n_q][n_q_heads][head_dim] of cfg.dtype
 *   out_dev : float [sum n_q][n_q_heads][head_dim]
 *   scale   : multiplies q.k before the softmax (1/sqrt(head_dim) in the paper) */
int wgkv_attend(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                const int32_t *n_q_host, const void *q_dev, const void *k_chunk_dev,
                const void *v_chunk_dev, const float *g_chunk_dev, float tau, float scale,
                float *out_dev, void *workspace_dev, size_t workspace_bytes, wgkv_stream stream);

/* Optional tuning of the decode form of wgkv_attend to the machine.  The tiles of a launch are
 * split evenly over its waves except for one correction: blocks go to the 8 XCDs of the GPU in
 * turn, and the odd XCD of each pair streams a few per cent slower than the even one, by an amount
 * that differs between machines.  This call runs the decode attention of every layer for the
 * given sequences (arguments as for wgkv_attend, the same queries for every layer; the cache is
 * not changed, out_dev is overwritten) with the correction set to 0, 2.5, 5, ... 12.5 per cent,
 * five timed passes over the layers each, and keeps the one with the lowest median for all later
 * calls on this pool (the default of 5 per cent unless another value is at least one per cent
 * faster).  Call it once, on a cache of the size the pool will serve; it synchronises with the
 * stream after every launch (30 passes: tens of milliseconds).  The outputs of later calls differ between
 * settings by the order of the floating-point sums only; for one setting they repeat bit for bit.
 *   skew_permille_out : optional, the value kept, in thousandths
 * Errors: INVALID_ARG, WORKSPACE, HIP. */
int wgkv_tune_decode_attention(wgkv_pool *pool, int32_t n_seqs, const int32_t *seq_ids_host,
                               const void *q_dev, float scale, float *out_dev, void *workspace_dev,
                               size_t workspace_bytes, wgkv_stream stream, int32_t *skew_permille_out);

/* For callers that cannot allocate or pass a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the decode form of wgkv_attend, same
 * arguments and same result, with the split-K partial results kept in an array of
 * WGKV_STATIC_SCRATCH_BYTES bytes that is part of the library's device image instead of in a
 * workspace.  Every GPU the library is loaded on holds its own copy until the process ends;
 * its address is looked up once per device by wgkv_init_pool.  The call allocates and frees
 * nothing and asks the runtime for nothing but the current device and the launch.
 *   q_dev [n_seqs][n_q_heads][head_dim] of cfg.dtype, out_dev float [n_seqs][n_q_heads][head_dim]
 * The launch uses at most 512 blocks, and the partials of that many blocks plus one per
 * (sequence, kv head) must fit: (2048 + n_seqs * n_kv_heads) * group * (head_dim + 2) * 4 bytes
 * (+ 256) <= WGKV_STATIC_SCRATCH_BYTES, else WGKV_ERR_WORKSPACE (every shape with group *
 * head_dim <= 512 fits at the largest call; use wgkv_attend otherwise).  Nothing in the array
 * has to start at zero (a partial is written before the count that announces it moves).  All
 * calls on one GPU share the array: two such calls that overlap in time on the same GPU, on
 * different streams or pools, race; calls in stream order do not.
 * Errors: INVALID_ARG, WORKSPACE, HIP (also: no pool was initialised on the current device). */
#define WGKV_STATIC_SCRATCH_BYTES (8u << 20)
int wgkv_attend_decode_static(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                              const void *q_dev, float scale, float *out_dev, wgkv_stream stream);

/* ---- read-time page selection over the admitted cache ----
 * Appendix "Synergy with KV Selection": Quest-style selection with key landmarks (the
 * per-page minimum and maximum key vectors) at a budget of so many KVs per query.  The
 * paper names the method only; this is the published Quest procedure as read here for
 * grouped-query attention: the criticality of page p of a kv head's global cache is
 *   U_p = max over the query heads g of the group of sum_e max(q_g[e] lo_p[e], q_g[e] hi_p[e]),
 * an upper bound of every q_g . K_j in the page; the min(n_pages, budget_pages) pages
 * with the largest U (total order of the fp32 bit patterns, equal scores: lower page
 * index first) are read, one selection per kv head; the local window is always read.
 *
 * Landmarks live in a caller-owned device buffer of wgkv_quest_landmark_bytes bytes,
 * zero-filled by the caller before its first use: per (slot, layer, kv head), in that
 * order, max_global_pages_per_head pages in cache order, each the minimum and the maximum
 * row in the pool dtype (2 * head_dim elements); then one int32 per (slot, layer, kv head).
 * The buffer grows with max_global_pages_per_head, not with the pool: 1 / page_size of
 * the keys of a cache in which every head is full.  It must be 16-byte aligned. */
int wgkv_quest_landmark_bytes(const wgkv_config *cfg, size_t *landmark_bytes);

/* Brings the landmarks of the given sequences' heads (layer `layer`) up to date with
 * their global caches: only pages that received entries since the last update are
 * recomputed.  reset != 0 recomputes all their pages; that is needed after
 * wgkv_evict_apply (entries moved) and after wgkv_free_seq (slot reused).  Call it after
 * the prefill / decode calls and before wgkv_quest_select.  Errors: INVALID_ARG, HIP. */
int wgkv_quest_update(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                      void *landmarks_dev, size_t landmark_bytes, int32_t reset, wgkv_stream stream);

/* Scores every page of every head for the decode queries and picks the pages to read.
 *   q_dev [n_seqs][n_q_heads][head_dim] of cfg.dtype, 16-byte aligned
 *   page_scores_out_dev float [n_seqs * n_kv_heads][score_stride]: U of pages [0, n_pages);
 *                       score_stride must cover the host's bound of every head's page count;
 *                       where the cache on the device is longer than the host knows (decode
 *                       steps replayed in a graph since the last wgkv_status), pages from
 *                       score_stride on are neither scored nor selected
 *   sel_pages_out_dev int32 [n_seqs * n_kv_heads][budget_pages]: ascending indices into the
 *                       head's global page table; sel_count_out_dev int32 [n_seqs * n_kv_heads]
 * fp32 arithmetic.  Errors: INVALID_ARG, HIP. */
int wgkv_quest_select(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                      const void *q_dev, void *landmarks_dev, size_t landmark_bytes, int32_t budget_pages,
                      float *page_scores_out_dev, int64_t score_stride, int32_t *sel_pages_out_dev,
                      int32_t *sel_count_out_dev, wgkv_stream stream);

/* Decode attention (as wgkv_attend with one query per sequence) over the local window and,
 * per kv head, only the listed pages of its global cache.
 *   sel_pages_dev int32 [n_seqs * n_kv_heads][sel_stride], strictly ascending page indices;
 *   sel_count_dev int32 [n_seqs * n_kv_heads].  Indices outside a head's table are clamped
 *   (the result is then meaningless but no memory outside the pool is read).
 * Errors: INVALID_ARG, WORKSPACE, HIP. */
int wgkv_attend_selected(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                         const void *q_dev, const int32_t *sel_pages_dev, const int32_t *sel_count_dev,
                         int32_t sel_stride, float scale, float *out_dev, void *workspace_dev,
                         size_t workspace_bytes, wgkv_stream stream);

/* Appendix "Eviction policy implementation", the three scoring steps, for every kv head
 * of the given sequences (distinct ids) over the N entries of its global cache:
 *   A = Softmax(Q_obs K^T * scale) per query row (n_obs positions x the heads of the group),
 *   S_raw[j] = sum over positions of the maximum over the group of A[.][j],
 *   S = MaxPool(S_raw, pool_w) along the cache order.
 * Readings: K is the global cache alone (the only entries eviction can take; all of them
 * are older than the window, so no mask applies) and each softmax is normalised over
 * these N entries; the pooling window is centred and clipped at both ends; pool_w odd.
 *   q_obs_dev : [n_seqs][n_obs][n_q_heads][head_dim] of cfg.dtype, the queries of the
 *               last n_obs positions of each sequence (the caller keeps them)
 *   scores_raw_out_dev, scores_out_dev : two distinct float buffers [n_seqs * n_kv_heads][stride];
 *               entries [0, N) of each row are written, the rest is left alone; stride must
 *               cover the host's upper bound of every head's length (see wgkv_status)
 * fp32 arithmetic; sums run in a fixed order, so the result repeats run to run.  The
 * workspace from wgkv_query_sizes covers n_obs <= 256 (n_units * n_obs * group * 8 bytes
 * are needed); n_obs <= 4096, pool_w <= 255, the group size must divide 64.
 * Errors: INVALID_ARG, WORKSPACE, HIP. */
int wgkv_evict_scores(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                      const void *q_obs_dev, int32_t n_obs, float scale, int32_t pool_w,
                      float *scores_raw_out_dev, float *scores_out_dev, int64_t stride,
                      void *workspace_dev, size_t workspace_bytes, wgkv_stream stream);

/* Appendix "Eviction policy implementation", the removal step: every kv head of the
 * given sequences (distinct ids) drops the floor(frac * N) entries of its global cache
 * with the lowest scores, N its current length ("the bottom 10 %": frac = 0.1; each
 * head on its own).  Scores are compared in the total order of their fp32 bit patterns;
 * among equal scores the older entry goes first.  The survivors keep their order and
 * are packed to the front in place; pages left without an entry return to the free
 * stack, units in (position in the call, kv head) order, a unit's pages in ascending
 * table index.  When to call it (the memory budget) is the caller's policy.
 *   scores_dev : float [n_seqs * n_kv_heads][stride], entry j of the head at
 *                [(b * n_kv_heads + h) * stride + j]; stride must cover the host's
 *                upper bound of every head's length (wgkv_status makes it exact); a head
 *                whose cache on the device is longer than stride (decode steps replayed
 *                in a graph since the last wgkv_status) is left as it is, and
 *                wgkv_evict_scores writes no score past the end of a row
 *   n_evicted_out_dev : optional int32 [n_seqs * n_kv_heads]
 * Errors: INVALID_ARG, WORKSPACE, HIP. */
int wgkv_evict_apply(wgkv_pool *pool, int32_t layer, int32_t n_seqs, const int32_t *seq_ids_host,
                     const float *scores_dev, int64_t stride, float frac,
                     int32_t *n_evicted_out_dev, void *workspace_dev, size_t workspace_bytes,
                     wgkv_stream stream);

/* Returns every page of a sequence slot to the free stack (layers ascending, kv
 * heads ascending, a unit's local pages then its global pages) and clears it. */
int wgkv_free_seq(wgkv_pool *pool, int32_t seq_id, wgkv_stream stream);

/* Synchronises the stream, reads free_top, the error flag, all token counts and all
 * global lengths back, and replaces the host-side bookkeeping (worst-case bounds, token
 * counts) by the exact values of the device.  Returns WGKV_ERR_DEVICE_FLAG when the device
 * flag is set (the bookkeeping has been refreshed all the same: a device-side refusal
 * changes no state), else WGKV_OK. */
int wgkv_status(wgkv_pool *pool, wgkv_stream stream, int64_t *pages_free,
                int32_t *device_error_flag);

/* Sec. 4.1 pool.  Clears the sticky device error flag, in stream order (one small kernel, so
 * the call may also be captured).  The flag is set by a kernel that found no free page or a
 * full page-table row (only replayed graphs get that far: direct calls are refused on the
 * host) and left all state as it was; once pages are back (wgkv_free_seq, wgkv_evict_apply)
 * the pool is usable again after this call and a wgkv_status.  Errors: INVALID_ARG, HIP. */
int wgkv_clear_error(wgkv_pool *pool, wgkv_stream stream);

/* Measurement aid: when both are non-NULL hipEvent_t handles, every later
 * wgkv_attend times its main attention kernel on the call's stream.  The decode
 * form attaches the two events to the kernel's own dispatch (hipExtLaunchKernelGGL:
 * they carry the begin and end time stamps of that dispatch, what a kernel trace
 * reports); the prefill form records ev_begin right before and ev_end right after
 * its kernels.  Pass NULLs to switch it off. */
int wgkv_set_profile_events(wgkv_pool *pool, void *ev_begin, void *ev_end);

/* Measurement aid: enqueues a kernel that reads bytes (rounded down to a multiple of 16) of
 * buf_dev (16-byte aligned) once, with the same kind of loads the decode attention kernel
 * streams K/V rows with, and does nothing else: its duration is what the memory system of
 * this machine gives a pure read of that size.  sink_dev: one uint32 the kernel may write.
 * When both are non-NULL hipEvent_t handles, ev_begin and ev_end take the begin and end time
 * stamps of the kernel's dispatch.  Errors: INVALID_ARG, HIP. */
int wgkv_stream_read_probe(const void *buf_dev, size_t bytes, uint32_t *sink_dev, void *ev_begin, void *ev_end,
                           wgkv_stream stream);

/* Frees the host handle only. */
void wgkv_destroy(wgkv_pool *pool);

/* Library version string (static storage). */
const char *wgkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WGKV_H */
