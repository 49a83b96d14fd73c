// Internal launch interface between the C ABI layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace sx {

// out[m][n] = sum_k act[m][k] * w[n][k] for a weight matrix given as up to three
// row blocks (q/k/v or gate/up share one launch).  Results are written as split-K
// partial sums  partial[ks][v][n]  with v = m * planes + plane: consumers add the
// ksplit * planes slices.  In head mode (V >= 0) rows n < V enter a fused argmax and
// rows V.. are the signal rows of the widened head.
// Rotary embedding + cache write done by the q/k/v projection's reducing epilogue (epi = 2):
// row r of the step is sequence r / W, rotary position pos[r / W] + level, cache entry
// pos[r / W] + node[r % W] (node null: the entry at pos).
struct RopeArgs {
  const int32_t* pos;
  int level;
  const int32_t* node;
  int W;
  float theta;
  double inv_freq[64];       // theta^(-2c/d) for c < d/2, filled on the host
  int Hq, Hkv, d;
  void* q_out;               // [rows][Hq][d] bf16
  int paged;
  void *kc, *vc;
  const int32_t* page_table;
  int page_size, max_pages;
  int64_t l_max;
  int64_t n_pages;           // paged: pages in the pool (page ids are forced into it)
  int* status;               // device error word or nullptr
};

// MFMA GEMM, activation pieces in LDS: one row of 16-byte entries per 8-wide k piece, one entry per
// virtual activation row v.  With 16 or more virtual rows the distance between the rows is a
// multiple of 16 entries and row v of k piece q sits at entry v ^ gemm_lds_swizzle(planes, q).
// That keeps both access patterns free of bank conflicts (measured with single-wave timing loops:
// 29.9 clocks per ds_write_b128 against 40.4 unswizzled, operand reads at the floor of 19.3):
// the staging writes, where eight neighbouring lanes hold two activation rows x four k pieces,
// and the operand reads, where 16 lanes hold 16 neighbouring rows of one k piece and the hardware
// pairs halves of neighbouring 16-lane groups.
__host__ __device__ inline int gemm_lds_row_stride(int Mv) { return Mv < 16 ? Mv : (Mv + 15) & ~15; }
__host__ __device__ inline int gemm_lds_swizzle(int Mv, int planes, int q) {
  if (Mv < 16) return 0;
  return planes == 1 ? 2 * q : ((q & 1) | ((q & 2) << 1));
}

struct GemmArgs {
  const void* w[3];
  int seg_end[3];      // exclusive end row of each block in the concatenated row space
  int nseg;
  int N, K, M;
  int planes;          // MFMA path: 1 = activations exact in bf16, 2 = bf16 hi + lo parts
  int ksplit;          // number of K ranges
  int kb_per_split;    // MFMA path: 128-element K blocks per range
  int spread;          // MFMA path, one K range, plain partial output (epi 0): workgroups to spread the 16-row tiles over in
                       // equal shares (each gets fewer than 8, its spare waves idle), or 0: 8 tiles per workgroup
  const float* act;    // VALU path: fp32 [M][K]
  // MFMA path: where the activations come from
  int a_mode;          // 0: fp32 rows [M][K]; 1: bf16 rows [M][K];
                       // 2: bf16 [embed[tok[m]] ; hidden[m]], each K/2 wide (the draft's fuse input)
                       // 3: RMSNorm of fp32 rows: a_src[m][k] * rsqrt(sum_j a_ssq[m][j] / K + a_eps) * a_gain[k]
                       // 4: silu(gate) * up, gate = columns k, up = columns K + k of the a_nslices
                       //    partial slices a_src left by a GEMM with N = 2K
  const void* a_src;   // rows (modes 0, 1, 3), hidden rows (mode 2) or partial sums (mode 4)
  const float* a_ssq;  // mode 3: [M][a_nssq] pieces of the rows' sums of squares
  int a_nssq;
  const void* a_gain;  // mode 3: [K] bf16 norm gain
  float a_eps;
  int a_nslices;       // mode 4: ksplit * planes of the producing GEMM
  int a_src_planes;    //         and its planes
  const void* a_embed; // mode 2: embedding table [V][K/2]
  const int32_t* a_tok;  // mode 2: token ids [M], forced into 0 .. a_vocab-1
  int a_vocab;
  int* status;         // device error word or nullptr (first out-of-range token id seen)
  int kc;              // K elements of activations staged in LDS at a time (multiple of 128)
  int wide;            // head mode over more than 32 bf16 rows: the kernel of gemm_wide.hip (weights through an LDS
                       // ring, activations in registers); head_wide_groups() candidates per row
  int wide_w;          //   its workgroups (each walks an equal share of the weight tiles)
  int wide_slots;      //   candidate slots per workgroup and row
  void* a_packed;      //   scratch of head_wide_pack_bytes() for the activations in operand order
  float* partial;      // [ksplit][M*planes][N] fp32, or nullptr in head mode
  // epi = 1: the workgroup that finishes a 128-row group last adds up the group's partial
  // sums in a fixed order (+ residual) and writes the finished rows
  int epi;
  int* counters;       // [groups], zero before the launch and again after it
  const float* residual;  // [M][N] or nullptr
  float* out_x;        // [M][N] fp32
  void* out_store;     // [M][N] bf16 or nullptr
  float* out_ssq;      // [M][groups] sum of squares of the group's columns, or nullptr
  RopeArgs rope;       // epi = 2: the finished rows are q / k / v heads (bf16 outputs)
  int V;               // head mode when >= 0
  int n_extra;
  int top_b;           // head mode: candidates kept per tile (0 or 1 = the argmax only)
  float* part_val;     // head mode: [M][ntiles][top_b] best values per 16-row tile, best first
  int* part_idx;       //            [M][ntiles][top_b] their row indices (INT_MAX = none)
  float* extra_out;    // [M][n_extra] or nullptr
  float* logits_dbg;   // [M][V] or nullptr
};

// Row-streaming GEMV for steps of at most four rows (gemv.hip): no split over K, the
// epilogue runs in the wave that owns a pair of weight rows.
struct GemvArgs {
  const void* w[3];
  int seg_end[3];
  int nseg;
  int N, K, M;
  int a_mode;            // as GemmArgs: 0 fp32 rows, 1 bf16 rows, 2 [embed[tok] ; hidden], 3 RMSNorm of fp32 rows
  const void* a_src;
  const void* a_embed;
  const int32_t* a_tok;  // mode 2: token ids [M], forced into 0 .. a_vocab-1
  int a_vocab;
  int* status;           // device error word or nullptr
  const float* a_ssq;
  int a_nssq;
  const void* a_gain;
  float a_eps;
  int epi;               // 0: rows (2p, 2p+1) -> residual add, out_x / out_store / out_ssq
                         // 1: rotary pairs of the q|k|v projection -> q_out / cache entries
                         // 2: (gate p, up p) of the gate|up projection -> out_x[m][p] = silu(gate) * up
                         // 3: widened head: rows < V -> per-workgroup argmax candidates part_val / part_idx
                         //    [M][grid], rows V.. -> extra_out [M][n_extra]; N may be odd
  const float* residual;
  float* out_x;
  void* out_store;
  float* out_ssq;        // [M][grid]
  int V, n_extra;        // epi 3
  float* part_val;
  int* part_idx;
  float* extra_out;
  RopeArgs rope;
  int stream;            // 1: weights read with non-temporal loads (read once; always for the head), 0: ordinary loads
  int grid, waves;       // launch shape, from gemv_plan
};
bool gemv_supported(int M, int N, int K);
size_t gemv_lds_bytes(const GemvArgs& g);
void gemv_plan(GemvArgs& g, int num_cus, int per_cu = 3);   // at most per_cu workgroups per compute unit
hipError_t launch_gemv(const GemvArgs& g, hipStream_t s);

inline int gemm_ntiles(int N) { return (N + 15) / 16; }
inline int gemm_groups(int N) { return (gemm_ntiles(N) + 7) / 8; }   // 128-row groups = workgroups along N
hipError_t launch_zero_i32(int* p, int n, hipStream_t s);
inline int gemm_mt(int M, int planes) { return (M * planes + 15) / 16; }

bool gemm_mfma_supported(int M, int planes, int K);
void choose_ksplit(GemmArgs& g, bool mfma, int num_cus);
hipError_t launch_gemm_valu(const GemmArgs& g, bool bf16, hipStream_t s);
hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s);
bool head_wide_supported(const GemmArgs& g);
void head_wide_plan(GemmArgs& g, int num_cus);   // sets wide, wide_w, wide_slots
int head_wide_groups(const GemmArgs& g);      // candidates per activation row
size_t head_wide_pack_bytes(const GemmArgs& g);
hipError_t launch_head_wide(const GemmArgs& g, hipStream_t s);
// reduce per-tile partial argmaxes: one result per activation row
// (with `sig` set it also applies the signal activations to extra[M][3]: the draft head's epilogue)
hipError_t launch_argmax_finalize(const float* part_val, const int* part_idx, int ntiles, int M,
                                  int32_t* argmax, float* max_logit, hipStream_t s,
                                  const float* extra = nullptr, int rem_activation = 0,
                                  float* sig_raw = nullptr, float* sig = nullptr);
// the top_b best per row, best first, from per-tile candidates (idxs given; C pairs per row)
// or from full rows of logits (idxs null; C = V values per row); rows lie `stride` apart
hipError_t launch_topb_finalize(const float* vals, const int* idxs, int C, int stride, int top_b, int M,
                                int32_t* cand_tok, float* cand_logit, hipStream_t s,
                                const float* extra = nullptr, int rem_activation = 0,
                                float* sig_raw = nullptr, float* sig = nullptr);
// VALU head path: logits [M][N] -> argmax over n < V, copy of signal rows and of logits
hipError_t launch_argmax_rows(const float* logits, int M, int N, int V, int n_extra,
                              int32_t* argmax, float* max_logit, float* extra_out,
                              float* logits_dbg, hipStream_t s);
// storage-type rows -> fp32 rows (ALU GEMM path only)
hipError_t launch_unpack_rows(const void* src, bool bf16, int M, int K, float* act, hipStream_t s);

// ---- attention -------------------------------------------------------------------------
struct AttnArgs {
  int dtype;                 // 0 fp32, 1 bf16
  int paged;
  const void *k, *v;
  const int32_t* page_table;
  int page_size, max_pages;
  int64_t l_max;
  int B, n_q, Hq, Hkv, d;
  const void* q;             // [B, n_q, Hq, d]
  const int32_t* ctx_len;    // [B] number of context entries before the block
  const uint64_t* mask;      // [B, n_q] or nullptr = chain
  int n_blk;                 // block entries stored after the context (normally n_q; tree drafting:
                             // every node written so far, of which n_q are this call's queries)
  int mask_stride;           // mask words between two sequences' rows (n_q; 0 = all sequences share)
  float scale;
  void* out;                 // [B, n_q, Hq, d] in dtype
  int wgrid;                 // workgroups of the split kernel; the keys of all (sequence, KV head) units
                             // are dealt to them in equal shares on the device (attn_sched.hpp)
  float* part_o;             // [wgrid + B*Hkv slots][R][d]
  float* part_ml;            // [wgrid + B*Hkv slots][R][2]  (running max, sum)
  int* sched;                // [B + 2] written by the split kernel for the merging kernel: prefix sums of the
                             // sequences' granule counts, then the number of workgroups that took part
  int64_t n_pages;           // paged: pages in the pool (page ids are forced into it)
  int* status;               // device error word or nullptr: first out-of-range length / page id seen
  int stages;                // matrix-core kernel: slots per tile ring (attn_plan)
  int use_mfma;              // matrix-core kernel (bf16, head_dim 128); its maxima are in log2 units
};
bool attn_mfma_supported(const AttnArgs& a);
size_t attn_mfma_lds_bytes(const AttnArgs& a);  // dynamic LDS of the matrix-core kernel as planned
int attn_mfma_per_cu(const AttnArgs& a);        // its workgroups per compute unit
int attn_mfma_stages(const AttnArgs& a);        // and slots per tile ring
int attn_mfma_max_chunk(const AttnArgs& a);   // longest chunk the matrix-core kernel takes
int attn_slots(const AttnArgs& a);            // partial-result slots a launch can write
hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s);
bool attn_plan(AttnArgs& a, int num_cus);      // false: the problem is outside what one launch can split
size_t attn_workspace_bytes(const AttnArgs& a);
void attn_carve(AttnArgs& a, void* workspace);   // points part_o / part_ml / sched into a workspace of that size
// hook(id, 0 / 1, stream) is called right before / after the split-KV kernel's launch
typedef void (*KernelHook)(int id, int phase, hipStream_t s);
hipError_t launch_attn(const AttnArgs& a, hipStream_t s, KernelHook hook = nullptr, int hook_id = 0);

// ---- draft-step glue kernels -----------------------------------------------------------
struct DraftDims {
  int dtype, D, Hq, Hkv, d, I, V;
  float rms_eps, rope_theta;
  int rem_activation;
};
hipError_t launch_embed_concat(const DraftDims& dm, int B, const void* embed, const int32_t* tok,
                               const void* hidden_in, float* act, hipStream_t s, int* status = nullptr);
// v[b][:] = residual[b][:] + sum of partial slices; optional copy to `sum_out` (fp32) and
// `hidden_out` (storage type); then RMSNorm with gain -> act (fp32)
hipError_t launch_reduce_norm(const DraftDims& dm, int B, int N, const float* partial, int nslices,
                              int planes, const float* residual, const void* gain, float* sum_out,
                              void* hidden_out, float* act, hipStream_t s);
// rows r = b * W + w: rotary position pos[b] + level, cache entry pos[b] + node[w] (node null: pos[b])
hipError_t launch_rope_kvwrite(const DraftDims& dm, int M, int W, const float* partial, int nslices,
                               int planes, const int32_t* pos, int level, const int32_t* node, void* q_out,
                               int kv_paged, void* kc, void* vc, const int32_t* page_table, int page_size,
                               int max_pages, int64_t l_max, hipStream_t s, int64_t n_pages = 0x7fffffff,
                               int* status = nullptr);
hipError_t launch_silu_mul(const DraftDims& dm, int B, const float* partial, int nslices, int planes,
                           float* act, hipStream_t s);
hipError_t launch_head_finalize(const DraftDims& dm, int B, const int32_t* argmax_in,
                                const float* extra, int32_t* next_tok, float* sig_raw, float* sig,
                                hipStream_t s);

// ---- measurement aid: copy of known size through the streaming load path -------------------
hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, bool nontemporal, hipStream_t s);

// ---- cache compaction after acceptance ---------------------------------------------------
struct CompactArgs {
  int paged;
  void *k, *v;
  const int32_t* page_table;
  int page_size, max_pages;
  int64_t l_max;
  int64_t n_pages;           // paged: pages in the pool (page ids are forced into it)
  int64_t layer_stride_bytes;
  int n_layers, B, n_q, Hkv;
  int row_bytes;             // head_dim * element size
  const int32_t *ctx_len, *accept_path, *accept_len, *last_node;
  int* status;               // device error word or nullptr
  const void* block_hidden;  // [B][n_q][hidden_row_bytes] or nullptr
  void* hidden_next;         // [B][hidden_row_bytes]
  int hidden_row_bytes;
};
bool kv_compact_supported(const CompactArgs& a);
hipError_t launch_kv_compact(const CompactArgs& a, hipStream_t s);

// ---- tree drafting: hand tokens and hidden states from one level to the next ----------------
struct TreeGatherArgs {
  int B, W_prev, top_b, W_next, n_q;
  int row_bytes;               // D * element size
  const int32_t *src_row, *rank, *node;   // [W_next]
  const int32_t* cand_tok;     // [B][W_prev][top_b]
  const void* hidden_prev;     // [B][W_prev][row_bytes]
  int32_t* tok_next;           // [B][W_next]
  void* hidden_next;           // [B][W_next][row_bytes] or nullptr
  int32_t* block_tok;          // [B][n_q] or nullptr
};
hipError_t launch_tree_gather(const TreeGatherArgs& a, hipStream_t s);

// ---- controller ------------------------------------------------------------------------
constexpr int kSmoothWords = 48;   // 3 signals x 16 words
struct ExitArgs {
  float alpha, thr_conf, thr_prog, thr_rem;
  uint32_t signal_mask;
  int smoother, window, split_pick, check_root, stop_think_token;
  int B, n_q, S;
  const int32_t *block_tok, *parent, *target_argmax;
  const float* sig;
  const int32_t *ctx_len, *split_tok;
  float* ewma;
  int32_t *n_obs, *is_thinking;
  float* smooth_state;       // [B][kSmoothWords] history of the window / momentum / paragraph smoothers
  int32_t *accept_len, *accept_path, *recover_tok, *last_node, *exit_flag, *new_ctx_len;
};
hipError_t launch_accept_exit(const ExitArgs& a, hipStream_t s);

}  // namespace sx
