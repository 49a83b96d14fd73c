/* specexit.h - C ABI of the SpecExit decode-round hot path for AMD MI355X (gfx950).
 *
 * One decode round of SpecExit (arXiv 2509.24248, Algorithm 1) is, per sequence:
 *   k x  specexit_draft_step      draft ("MTP") forward with the widened head (Sec. 3.1, Eq. 1)
 *   1 x  specexit_verify_attn     target attention over [last accepted | draft candidates]
 *                                 with tree attention (Alg. 1), once per target layer
 *   1 x  specexit_lmhead_argmax   target logits -> recover / verification tokens (Alg. 1)
 *   1 x  specexit_accept_exit     acceptance, signal smoothing, stop thresholds and the
 *                                 step-split exit (Alg. 1; Sec. 3.3; Appendix)
 *
 * Conventions
 *   - Every array argument is a DEVICE pointer owned by the caller unless marked [host].
 *     Descriptor structs are host structs read at call time; their first field is
 *     struct_size = sizeof(the struct) as compiled by the caller.
 *   - Calls only enqueue kernels on `stream` (a hipStream_t passed as void*; NULL = the
 *     default stream).  They never allocate or free device memory, never synchronise and
 *     never copy to the host, so a round may be captured in a HIP graph by the caller.
 *   - Scratch memory is the caller's `workspace` (256-byte aligned), at least as large as
 *     the matching *_workspace_bytes() query says.  Its contents are undefined afterwards.
 *   - Return value: SPECEXIT_OK or a negative error code; specexit_last_error() then
 *     returns a thread-local description.  No kernel is launched when validation fails.
 *   - Contents of device arrays never reach an address unchecked: context lengths, cache
 *     positions, page ids, token ids and node ids are forced into their valid range before use,
 *     so a bad value gives a wrong result for its sequence or row and never a memory fault.
 *     With SPECEXIT_FLAG_VALIDATE in `flags` the first such value seen by a call's kernels is
 *     also reported in the device status word registered with specexit_set_dev_status.
 *   - dtype selects the storage type of weights, KV caches, q, hidden states and the
 *     attention output (SPECEXIT_F32 or SPECEXIT_BF16).  Accumulation, softmax, norms and
 *     activations are always fp32.  All matrices are row-major [out, in].
 */
#ifndef SPECEXIT_H
#define SPECEXIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPECEXIT_OK            0
#define SPECEXIT_EINVAL       (-1)  /* null pointer, bad size, inconsistent shapes            */
#define SPECEXIT_EUNSUPPORTED (-2)  /* shape or type outside what the kernels implement       */
#define SPECEXIT_EWORKSPACE   (-3)  /* workspace missing, misaligned or too small             */
#define SPECEXIT_ELAUNCH      (-4)  /* the HIP runtime refused a launch                       */

typedef enum { SPECEXIT_F32 = 0, SPECEXIT_BF16 = 1 } specexit_dtype;
typedef enum { SPECEXIT_KV_CONTIG = 0, SPECEXIT_KV_PAGED = 1 } specexit_kv_layout;

/* Limits: 1 <= n_q <= 64 (one mask bit per block entry); head_dim in {64, 128};
 * n_q_heads % n_kv_heads == 0; (n_q_heads / n_kv_heads) * n_q <= 128;
 * page_size a multiple of 16; hidden, intermediate, n_q_heads*head_dim multiples of 64. */
/* flags bit: the workspace passed to specexit_draft_step / specexit_draft_tree_level was
 * zero-filled once (specexit_workspace_prepare) and has since been written only by calls of
 * that same entry point with the same descriptor, cache view and row counts.  The call then
 * skips the launch that clears its arrival counters (every kernel leaves them at zero). */
#define SPECEXIT_FLAG_WORKSPACE_PREPARED 1u
/* flags bit: report out-of-range device data.  The kernels of the call write the first problem
 * they see into the status word of the calling host thread (specexit_set_dev_status), if that
 * word is still 0: SPECEXIT_STATUS_*.  The call itself still returns SPECEXIT_OK (it does not
 * wait for its kernels); the caller reads the word when it synchronises, and zeroes it. */
#define SPECEXIT_FLAG_VALIDATE 2u
#define SPECEXIT_STATUS_OK         0
#define SPECEXIT_STATUS_BAD_LENGTH 1 /* ctx_len / pos negative or beyond the cache capacity       */
#define SPECEXIT_STATUS_BAD_PAGE   2 /* page id outside 0 .. n_pages-1                            */
#define SPECEXIT_STATUS_BAD_TOKEN  3 /* token id outside 0 .. vocab-1                             */
#define SPECEXIT_STATUS_BAD_NODE   4 /* node id / path entry outside its block                    */
#define SPECEXIT_MAX_NQ 64
#define SPECEXIT_MAX_TOP_B 4 /* ranked continuations a tree-drafting row can report */
#define SPECEXIT_N_SIGNALS 3

/* Registers (dev_status != NULL) or clears (NULL) the device int32 that calls made by THIS host
 * thread with SPECEXIT_FLAG_VALIDATE report into.  [host] call; the word itself is device memory
 * owned by the caller, zeroed by the caller, and must stay valid while such calls are in flight. */
int32_t specexit_set_dev_status(int32_t *dev_status);

/* Draft model dimensions (the draft layer mirrors the target's attention geometry). */
typedef struct {
  uint32_t struct_size;
  int32_t dtype;           /* specexit_dtype */
  int32_t hidden;          /* D */
  int32_t n_q_heads, n_kv_heads, head_dim;
  int32_t intermediate;    /* I, width of the gated MLP */
  int32_t vocab;           /* V; the head has V + 3 rows */
  float rms_eps;           /* RMSNorm epsilon */
  float rope_theta;        /* rotary base */
  int32_t rem_activation;  /* remaining-length head: 0 = max(0, expm1(z)) (inverse of the
                              log(1+r) training target, Eq. 5), 1 = sigmoid, 2 = identity */
} specexit_model_desc;

/* Draft weights, dtype = desc.dtype, row-major [out, in].  The three norm vectors are
 * also stored in dtype.  w_head rows: 0..V-1 = W_tok, V = W_conf, V+1 = W_prog,
 * V+2 = W_rem (Eq. 1). */
typedef struct {
  uint32_t struct_size;
  const void *embed;     /* [V, D]            */
  const void *w_fc;      /* [D, 2D]  applied to [embedding ; hidden_in] */
  const void *ln_attn, *ln_mlp, *ln_final; /* [D] */
  const void *w_q;       /* [Hq*d, D]         */
  const void *w_k, *w_v; /* [Hkv*d, D]        */
  const void *w_o;       /* [D, Hq*d]         */
  const void *w_gate, *w_up; /* [I, D]        */
  const void *w_down;    /* [D, I]            */
  const void *w_head;    /* [V+3, D]          */
} specexit_draft_weights;

/* One layer's K/V cache.
 *   CONTIG: k, v are [B, n_kv_heads, l_max, head_dim].
 *   PAGED : k, v are [n_pages, n_kv_heads, page_size, head_dim]; page_table is
 *           [B, max_pages_per_seq] int32; token t of sequence b lives in page
 *           page_table[b, t / page_size], slot t % page_size.  l_max is then
 *           max_pages_per_seq * page_size.
 * Table entries past a sequence's last used page are never read. */
typedef struct {
  uint32_t struct_size;
  int32_t layout;        /* specexit_kv_layout */
  int32_t dtype;
  int32_t n_kv_heads, head_dim;
  void *k, *v;
  const int32_t *page_table;
  int32_t page_size, max_pages_per_seq;
  int64_t l_max, n_pages;
} specexit_kv_view;

/* Exit controller settings.  Defaults of the paper: alpha 0.1 (Appendix, EWMA);
 * confidence > 0.8, progress > 0.3, remaining < 200 for the combined rule, or
 * 0.9 / 0.8 / 100 with a single bit of signal_mask (Appendix, "Stop Threshold"). */
typedef struct {
  uint32_t struct_size;
  float alpha, thr_conf, thr_prog, thr_rem;
  uint32_t signal_mask;    /* bit 0 confidence, 1 progress, 2 remaining; ANDed */
  int32_t smoother;        /* SPECEXIT_SMOOTH_*: 0 EWMA, 1 none, 2 sliding window, 3 momentum, 4 paragraph mean */
  int32_t split_pick;      /* 0 earliest step-split token in the accepted path, 1 latest */
  int32_t check_root;      /* 1: the block root may also act as the step-split token */
  int32_t stop_think_token;
  int32_t window;          /* N of the sliding-window and momentum smoothers, 1..16; 0 = the paper's 10 */
} specexit_exit_cfg;

/* Smoothers of the Appendix ("Signal Smoothing"). */
#define SPECEXIT_SMOOTH_EWMA      0
#define SPECEXIT_SMOOTH_NONE      1
#define SPECEXIT_SMOOTH_WINDOW    2
#define SPECEXIT_SMOOTH_MOMENTUM  3
#define SPECEXIT_SMOOTH_PARAGRAPH 4
/* 32-bit words of per-sequence history the smoothers 2..4 keep in smooth_state */
#define SPECEXIT_SMOOTH_WORDS 48

/* ---- stage 1: draft step (Sec. 3.1 Eq. 1; Sec. 3.2 Eqs. 3-5; Alg. 1, first loop line) ----
 * For each of the B rows: x = W_fc [embed[tok] ; hidden_in]; one pre-norm decoder layer
 * (RMSNorm, GQA attention with rotary embedding over the draft's own cache positions
 * 0..pos including the entry written now at pos, residual, RMSNorm, gated SiLU MLP,
 * residual) -> hidden_out; z = W_head RMSNorm(hidden_out); next_tok = argmax z[0:V]
 * (lowest index on ties); sig_raw = z[V:V+3]; sig = (sigmoid, sigmoid, rem_activation).
 * draft_kv is updated in place at position pos[b].  hidden_in/hidden_out are [B, D] in
 * dtype and may not alias.  1 <= B <= 64. */
int32_t specexit_draft_step(const specexit_model_desc *desc, const specexit_draft_weights *w,
                            const specexit_kv_view *draft_kv, int32_t B,
                            const int32_t *tok /*[B]*/, const void *hidden_in /*[B,D]*/,
                            const int32_t *pos /*[B]*/,
                            void *hidden_out /*[B,D]*/, int32_t *next_tok /*[B]*/,
                            float *sig_raw /*[B,3]*/, float *sig /*[B,3]*/,
                            void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);
size_t specexit_draft_step_workspace_bytes(const specexit_model_desc *desc,
                                           const specexit_kv_view *draft_kv, int32_t B);

/* ---- replaying a fixed sequence of calls (Alg. 1's round: draft steps, verification, head,
 * acceptance; the abstract's and Sec. 1's point is that exit detection must add no overhead to
 * the decode loop, and at batch 1 that loop is a chain of some sixty short launches) ----
 * specexit_graph_begin puts `stream` (not the null stream) into HIP stream capture; every call of
 * this library enqueued on it until specexit_graph_end is recorded instead of run, with the
 * pointers, sizes and flags passed then.  specexit_graph_end returns an executable graph that
 * specexit_graph_launch replays on any stream: all recorded kernels in their order, reading and
 * writing the same device buffers (which the caller keeps alive and may refill between
 * replays).  Each entry point must have been called once with the same shapes before the
 * capture (first calls set kernel attributes and query the device, which capture forbids), and
 * nothing else may use the stream or allocate device memory on this thread while capturing.
 * The graph owns no buffers; specexit_graph_destroy releases it.  Host pointers: `out` and the
 * graph handle.  Errors: SPECEXIT_EINVAL (null arguments), SPECEXIT_ELAUNCH (the runtime
 * refused; the capture is ended and dropped). */
typedef struct specexit_graph specexit_graph;
int32_t specexit_graph_begin(void *stream);
int32_t specexit_graph_end(void *stream, specexit_graph **out);
int32_t specexit_graph_launch(const specexit_graph *graph, void *stream);
int32_t specexit_graph_destroy(specexit_graph *graph);

/* Zero-fills a workspace (a small kernel on `stream`; see SPECEXIT_FLAG_WORKSPACE_PREPARED). */
int32_t specexit_workspace_prepare(void *workspace, size_t workspace_bytes, void *stream);

/* ---- stage 1 over a tree: one level of tree drafting (it builds the candidate block that the
 * target's verification forward of Alg. 1 checks; the draft forward is that of
 * specexit_draft_step) ----
 * The candidate tree has a fixed topology: node 0 is the last accepted token, node c > 0 holds
 * the rank[c]-th most likely continuation (0 = argmax) of its parent.  A level call runs the
 * draft forward for W nodes of equal depth `level` of each of the B sequences (rows ordered
 * [B, W]; B * W <= 64): row (b, w) has token tok[b,w], input hidden state hidden_in[b,w,:] (its
 * parent's hidden_out; the target's hidden state for node 0), rotary position ctx_len[b] + level,
 * its K/V are stored in draft cache entry ctx_len[b] + node[w], and it attends to the context
 * 0..ctx_len[b]-1 plus the block entries ctx_len[b] + j whose bit j is set in anc_mask[w]
 * (ancestors and itself; node and anc_mask are device arrays shared by all sequences).
 * Entries ctx_len[b] .. ctx_len[b] + n_blk - 1 must hold finite values once this call has
 * written its own (number the nodes level by level and pass n_blk = last node of this level
 * + 1).  Outputs per row: hidden_out, the top_b best tokens cand_tok[b,w,0:top_b] (logit
 * descending, lower index first among equals) with their logits cand_logit (may be NULL),
 * sig_raw and sig as in specexit_draft_step.  With W = 1, level = 0, node = {0}, anc_mask =
 * {1}, n_blk = 1, top_b = 1 this is specexit_draft_step at pos = ctx_len. */
int32_t specexit_draft_tree_level(const specexit_model_desc *desc, const specexit_draft_weights *w,
                                  const specexit_kv_view *draft_kv, int32_t B, int32_t W,
                                  const int32_t *tok /*[B,W]*/, const void *hidden_in /*[B,W,D]*/,
                                  const int32_t *ctx_len /*[B]*/, int32_t level,
                                  const int32_t *node /*[W]*/, const uint64_t *anc_mask /*[W]*/,
                                  int32_t n_blk, int32_t top_b,
                                  void *hidden_out /*[B,W,D]*/, int32_t *cand_tok /*[B,W,top_b]*/,
                                  float *cand_logit /*[B,W,top_b] or NULL*/,
                                  float *sig_raw /*[B,W,3]*/, float *sig /*[B,W,3]*/,
                                  void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);
size_t specexit_draft_tree_level_workspace_bytes(const specexit_model_desc *desc,
                                                 const specexit_kv_view *draft_kv, int32_t B,
                                                 int32_t W, int32_t top_b);

/* Between two levels: row wn of the next level is the child with rank rank[wn] of row
 * src_row[wn] of the level just computed: tok_next[b,wn] = cand_tok[b, src_row[wn], rank[wn]]
 * (also written to block_tok[b, node[wn]] when block_tok [B, n_q] is given) and
 * hidden_next[b,wn,:] = hidden_prev[b, src_row[wn], :] (skipped when hidden_next is NULL: leaves
 * need no forward).  src_row, rank, node are device arrays [W_next]. */
int32_t specexit_tree_gather(int32_t dtype, int32_t B, int32_t W_prev, int32_t top_b, int32_t W_next,
                             int32_t D, int32_t n_q, const int32_t *src_row, const int32_t *rank,
                             const int32_t *node, const int32_t *cand_tok /*[B,W_prev,top_b]*/,
                             const void *hidden_prev /*[B,W_prev,D]*/, int32_t *tok_next /*[B,W_next]*/,
                             void *hidden_next /*[B,W_next,D] or NULL*/, int32_t *block_tok /*[B,n_q] or NULL*/,
                             uint32_t flags, void *stream);

/* ---- stage 2: verification attention (Alg. 1, target verification step: the block's queries
 * under a chain or tree-ancestor mask) ----
 * out[b,i,h,:] = sum_j softmax_j(scale * q[b,i,h,:] . K[j]) V[j] over the visible cache
 * positions j of query i: the context 0..ctx_len[b]-1 plus the block entries
 * ctx_len[b]+t whose bit t is set in mask[b,i] (mask NULL = chain: bits 0..i).  The
 * block's K/V must already be stored at positions ctx_len[b] .. ctx_len[b]+n_q-1.
 * Query head h reads KV head h / (n_q_heads / n_kv_heads).  q and out are
 * [B, n_q, n_q_heads, head_dim] in kv->dtype.  Every mask row must have at least one
 * visible position (bit i of row i is normally set). */
int32_t specexit_verify_attn(const specexit_kv_view *kv, int32_t B, int32_t n_q, int32_t n_q_heads,
                             const void *q, const int32_t *ctx_len /*[B]*/,
                             const uint64_t *mask /*[B,n_q] or NULL*/, float scale, void *out,
                             void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);
size_t specexit_verify_attn_workspace_bytes(const specexit_kv_view *kv, int32_t B, int32_t n_q,
                                            int32_t n_q_heads);

/* ---- stage 3: LM head -> argmax (Alg. 1, the target's own next tokens that acceptance compares
 * against and recovers from; greedy) ----
 * z = hidden . w^T with w [V + n_extra, D]; argmax[r] = lowest index of the maximum of
 * z[r, 0:V].  Rows V.. of w (the widened head's signal rows, Eq. 1) never enter the
 * argmax; their products go to extra_out [M, n_extra].  max_logit, extra_out and
 * logits_dbg ([M, V] fp32, every logit; for tests) may be NULL.  1 <= M <= 144. */
int32_t specexit_lmhead_argmax(int32_t dtype, int32_t M, int32_t D, int32_t V, int32_t n_extra,
                               const void *hidden /*[M,D]*/, const void *w /*[V+n_extra,D]*/,
                               int32_t *argmax /*[M]*/, float *max_logit /*[M]*/,
                               float *extra_out /*[M,n_extra]*/, float *logits_dbg /*[M,V]*/,
                               void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);
size_t specexit_lmhead_argmax_workspace_bytes(int32_t dtype, int32_t M, int32_t D, int32_t V,
                                              int32_t n_extra);

/* ---- specexit_lmhead_argmax for callers that cannot allocate: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * specexit_lmhead_argmax, but no workspace: the scratch (the per-tile argmax candidates) lives in
 * a buffer built into the library, SPECEXIT_NOALLOC_SCRATCH_BYTES per GPU, held from the first
 * call on that GPU until the process ends.  The call allocates and frees nothing.  Shapes whose
 * scratch would not fit (the query specexit_lmhead_argmax_workspace_bytes says how much) are
 * refused with SPECEXIT_EWORKSPACE; 12 MiB covers every bf16 shape up to M = 144, V + n_extra =
 * 151952.  All calls on one GPU share that GPU's buffer: calls that overlap in time on one GPU
 * (two streams, two threads) race and must be ordered by the caller.  The buffer keeps the last
 * call's contents; nothing in it has to be cleared between calls.  The first call on a GPU looks
 * the buffer's address up and must therefore come before any stream capture. */
#define SPECEXIT_NOALLOC_SCRATCH_BYTES (12u << 20)
int32_t specexit_lmhead_argmax_noalloc(int32_t dtype, int32_t M, int32_t D, int32_t V, int32_t n_extra,
                                       const void *hidden /*[M,D]*/, const void *w /*[V+n_extra,D]*/,
                                       int32_t *argmax /*[M]*/, float *max_logit /*[M]*/,
                                       float *extra_out /*[M,n_extra]*/, float *logits_dbg /*[M,V]*/,
                                       uint32_t flags, void *stream);

/* ---- stages 4 + 5: acceptance, smoothing, exit rule (Alg. 1; Sec. 3.3; Appendix) ----
 * Per sequence b:
 *  smoothing  if is_thinking: x = sig on the first observation (n_obs == 0) or when
 *             smoother == 1, else x = alpha*sig + (1-alpha)*x; n_obs += 1.
 *             Smoothers 2..4 (Appendix, "Signal Smoothing") keep the observations in
 *             smooth_state: 2 = mean of the last N; 3 = forecast of the next score, the latest
 *             observation + mean of the N-1 differences between the last N; 4 = mean of all
 *             observations of the current paragraph, a paragraph ending in a round that accepts
 *             a step-split token without leaving thinking.  While fewer than N observations
 *             exist, 2 and 3 use those there are.  x is written to ewma in every mode.
 *  accept     walk from node 0: move to the lowest-index child c of the current node with
 *             block_tok[c] == target_argmax[current]; accept_path lists the nodes entered
 *             (-1 padded), accept_len their number, last_node the final node,
 *             recover_tok = target_argmax[last_node].  parent NULL = chain (parent i-1).
 *  exit       pass = AND over signal_mask of (x0 > thr_conf, x1 > thr_prog, x2 < thr_rem).
 *             If is_thinking and pass and an accepted draft token is in split_tok: the
 *             path is cut right after that token (earliest or latest per split_pick),
 *             recover_tok = stop_think_token, is_thinking = 0, exit_flag = 1.
 *  new_ctx_len = ctx_len + 1 + accept_len.
 * ewma [B,3], n_obs [B], is_thinking [B] are in/out state, and so is smooth_state
 * [B, SPECEXIT_SMOOTH_WORDS] (32-bit words, zero-filled by the caller when a sequence starts,
 * opaque afterwards; required for smoothers 2..4, may be NULL otherwise).  split_tok is
 * sorted ascending, S >= 0.  block_tok/parent/target_argmax are [B, n_q]. */
int32_t specexit_accept_exit(const specexit_exit_cfg *cfg, int32_t B, int32_t n_q,
                             const int32_t *block_tok, const int32_t *parent,
                             const int32_t *target_argmax, const float *sig /*[B,3]*/,
                             const int32_t *ctx_len /*[B]*/, const int32_t *split_tok, int32_t S,
                             float *ewma, int32_t *n_obs, int32_t *is_thinking,
                             float *smooth_state /*[B,SPECEXIT_SMOOTH_WORDS] or NULL*/,
                             int32_t *accept_len /*[B]*/, int32_t *accept_path /*[B,n_q]*/,
                             int32_t *recover_tok /*[B]*/, int32_t *last_node /*[B]*/,
                             int32_t *exit_flag /*[B]*/, int32_t *new_ctx_len /*[B]*/,
                             uint32_t flags, void *stream);

/* ---- after the round: cache compaction (Alg. 1, cache-update step inside the exit branch,
 * applied after every round) ----
 * Per sequence b, with L = ctx_len[b] (the value the round started with) and the outputs of
 * specexit_accept_exit: the K/V entry of accepted node accept_path[b,j], stored at cache
 * position L + accept_path[b,j] during verification, moves to position L + 1 + j for
 * j < accept_len[b] (the root stays at L), in every one of the n_layers caches that lie
 * layer_stride_bytes apart from kv->k / kv->v (all layers share kv's shape and, when
 * paged, its page table).  Entries past L + accept_len[b] are dead afterwards; nothing
 * else is written.  Every moved entry is read before any is written, so overlapping
 * source and target positions are safe.  With block_hidden [B, n_q, D] (in kv->dtype, the
 * target's final hidden states of the block) the row of last_node[b] is copied to
 * hidden_next [B, D], the input of the next round's first draft step; block_hidden NULL
 * skips that (last_node and hidden_next are then unused).  D * element size must be a
 * multiple of 16.  A sequence whose block does not fit the cache (L + n_q > l_max) is left
 * untouched. */
int32_t specexit_kv_compact(const specexit_kv_view *kv, int32_t n_layers, int64_t layer_stride_bytes,
                            int32_t B, int32_t n_q, const int32_t *ctx_len /*[B]*/,
                            const int32_t *accept_path /*[B,n_q]*/, const int32_t *accept_len /*[B]*/,
                            const int32_t *last_node /*[B]*/, const void *block_hidden /*[B,n_q,D] or NULL*/,
                            int32_t D, void *hidden_next /*[B,D]*/, uint32_t flags, void *stream);

/* ---- measurement aid -------------------------------------------------------------------
 * Hands the library n pairs of caller-owned hipEvent_t ([host] arrays of handles).  From then
 * on, each launch of the named kernel records the next unused pair around that one kernel (for
 * the ids called spans: around those consecutive launches of one call) on the call's stream
 * (start before, stop after), until the pairs run out; n = 0 disarms.
 * Returns the number of pairs consumed so far for that kernel when called with n < 0.
 * Arming and recording are serialised by a lock; do not arm while a stream is being captured
 * into a graph. */
#define SPECEXIT_PROF_DRAFT_HEAD_GEMM 0 /* widened-head GEMM + argmax inside specexit_draft_step */
#define SPECEXIT_PROF_LMHEAD_GEMM     1 /* GEMM + argmax inside specexit_lmhead_argmax            */
#define SPECEXIT_PROF_VERIFY_ATTN     2 /* split-KV kernel inside specexit_verify_attn            */
#define SPECEXIT_PROF_DRAFT_ATTN      3 /* split-KV kernel inside specexit_draft_step             */
#define SPECEXIT_PROF_DRAFT_PROJ_IN   4 /* span: fuse + q|k|v projections of specexit_draft_step  */
#define SPECEXIT_PROF_DRAFT_PROJ_OUT  5 /* span: o, gate|up (+ SiLU gate), down projections       */
#define SPECEXIT_PROF_COUNT           6
int32_t specexit_profile_events(int32_t kernel, void *const *start_events, void *const *stop_events,
                                int32_t n);

/* Copies `bytes` (a multiple of 16; both pointers 16-byte aligned, device memory, no overlap)
 * with 16-byte loads: non-temporal ones, as the weight and KV streams use, when nontemporal
 * != 0, ordinary ones otherwise.  A plain kernel of known traffic: profiler byte counters
 * read for the library's kernels are scaled by what they read for this one. */
int32_t specexit_copy_probe(const void *src, void *dst, size_t bytes, int32_t nontemporal, void *stream);

/* ---- scratch sizes, one query for every call ------------------------------------------------
 * Bytes of workspace that call `op` needs for B sequences and n_q block entries (draft tree level:
 * n_q = W rows per sequence; LM head: M = B * n_q rows).  `desc` is a [host] struct of the op's
 * query type below (first field struct_size); 0 is returned for shapes the call would reject and
 * for ops that use no scratch.  The per-call *_workspace_bytes functions give the same numbers. */
#define SPECEXIT_OP_DRAFT_STEP       0 /* desc: specexit_draft_query                        */
#define SPECEXIT_OP_VERIFY_ATTN      1 /* desc: specexit_attn_query                         */
#define SPECEXIT_OP_LMHEAD_ARGMAX    2 /* desc: specexit_lmhead_query                       */
#define SPECEXIT_OP_ACCEPT_EXIT      3 /* no scratch: 0                                     */
#define SPECEXIT_OP_DRAFT_TREE_LEVEL 4 /* desc: specexit_draft_query (top_b used)           */
#define SPECEXIT_OP_KV_COMPACT       5 /* no scratch: 0                                     */
typedef struct {
  uint32_t struct_size;
  const specexit_model_desc *desc;
  const specexit_kv_view *draft_kv;
  int32_t top_b; /* tree level only */
} specexit_draft_query;
typedef struct {
  uint32_t struct_size;
  const specexit_kv_view *kv;
  int32_t n_q_heads;
} specexit_attn_query;
typedef struct {
  uint32_t struct_size;
  int32_t dtype, hidden, vocab, n_extra;
} specexit_lmhead_query;
size_t specexit_workspace_bytes(int32_t op, const void *desc, int32_t B, int32_t n_q);

const char *specexit_last_error(void); /* [host] thread-local, never NULL */
uint32_t specexit_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SPECEXIT_H */
