// C ABI of the SpecExit decode-round library: argument checks, workspace carving and the
// order of kernel launches.  No arithmetic of the method lives here.
#include "../../include/specexit.h"

#include "common.hpp"
#include "kernels.hpp"

#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

using namespace sx;

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int32_t check_hip(hipError_t e, const char* what) {
  if (e == hipSuccess) return SPECEXIT_OK;
  return fail(SPECEXIT_ELAUNCH, "%s: %s", what, hipGetErrorString(e));
}

int num_cus() {
  // queried once per process (function-local static: initialised under the language's own lock)
  static const int n = [] {
    int dev = 0, cus = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess) cus = p.multiProcessorCount;
    return cus > 0 ? cus : 256;
  }();
  return n;
}

// device status word of this host thread (specexit_set_dev_status); used by calls that pass
// SPECEXIT_FLAG_VALIDATE
static_assert(kStatusBadLength == SPECEXIT_STATUS_BAD_LENGTH && kStatusBadPage == SPECEXIT_STATUS_BAD_PAGE &&
              kStatusBadToken == SPECEXIT_STATUS_BAD_TOKEN && kStatusBadNode == SPECEXIT_STATUS_BAD_NODE,
              "status codes of the ABI and of the kernels differ");
thread_local int32_t* g_dev_status = nullptr;
int* status_for(uint32_t flags) { return (flags & SPECEXIT_FLAG_VALIDATE) ? g_dev_status : nullptr; }

// caller-provided event pairs recorded around single kernels (measurement aid)
struct ProfSlot {
  std::vector<hipEvent_t> start, stop;
  size_t used = 0;
};
ProfSlot g_prof[SPECEXIT_PROF_COUNT];
std::mutex g_prof_mu;   // arming and recording may come from different host threads

struct ProfScope {
  ProfSlot* slot;
  hipStream_t s;
  bool on;
  std::unique_lock<std::mutex> lock;
  ProfScope(int id, hipStream_t st) : slot(&g_prof[id]), s(st), lock(g_prof_mu) {
    on = slot->used < slot->start.size();
    if (on) (void)hipEventRecord(slot->start[slot->used], s);
    else lock.unlock();
  }
  ~ProfScope() {
    if (on) {
      (void)hipEventRecord(slot->stop[slot->used], s);
      ++slot->used;
    }
  }
};

void g_prof_hook(int id, int phase, hipStream_t s) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  ProfSlot& sl = g_prof[id];
  if (sl.used >= sl.start.size()) return;
  if (phase == 0) {
    (void)hipEventRecord(sl.start[sl.used], s);
  } else {
    (void)hipEventRecord(sl.stop[sl.used], s);
    ++sl.used;
  }
}

size_t align256(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* p) : base(static_cast<char*>(p)) {}
  template <typename T> T* take(size_t bytes) {
    T* r = reinterpret_cast<T*>(base ? base + off : nullptr);
    off += align256(bytes);
    return r;
  }
};

bool dtype_ok(int32_t dt) { return dt == SPECEXIT_F32 || dt == SPECEXIT_BF16; }
size_t esize(int32_t dt) { return dt == SPECEXIT_BF16 ? 2 : 4; }

int32_t check_kv(const specexit_kv_view* kv, const char* who) {
  if (!kv || kv->struct_size != sizeof(specexit_kv_view)) return fail(SPECEXIT_EINVAL, "%s: kv view missing or of another ABI size", who);
  if (!dtype_ok(kv->dtype)) return fail(SPECEXIT_EINVAL, "%s: unknown kv dtype %d", who, kv->dtype);
  if (!kv->k || !kv->v) return fail(SPECEXIT_EINVAL, "%s: kv pointers are null", who);
  if (kv->head_dim != 64 && kv->head_dim != 128) return fail(SPECEXIT_EUNSUPPORTED, "%s: head_dim %d not in {64,128}", who, kv->head_dim);
  if (kv->n_kv_heads < 1) return fail(SPECEXIT_EINVAL, "%s: n_kv_heads < 1", who);
  if (kv->layout == SPECEXIT_KV_PAGED) {
    if (!kv->page_table) return fail(SPECEXIT_EINVAL, "%s: paged layout without page_table", who);
    if (kv->page_size < 16 || kv->page_size % 16) return fail(SPECEXIT_EUNSUPPORTED, "%s: page_size %d is not a multiple of 16", who, kv->page_size);
    if (kv->max_pages_per_seq < 1 || kv->n_pages < 1) return fail(SPECEXIT_EINVAL, "%s: empty page pool", who);
  } else if (kv->layout == SPECEXIT_KV_CONTIG) {
    if (kv->l_max < 1) return fail(SPECEXIT_EINVAL, "%s: l_max < 1", who);
  } else {
    return fail(SPECEXIT_EINVAL, "%s: unknown kv layout %d", who, kv->layout);
  }
  return SPECEXIT_OK;
}

int32_t fill_attn(AttnArgs& a, const specexit_kv_view* kv, int32_t B, int32_t n_q, int32_t n_q_heads, const char* who) {
  int32_t rc = check_kv(kv, who);
  if (rc) return rc;
  if (B < 1) return fail(SPECEXIT_EINVAL, "%s: B < 1", who);
  if (n_q < 1 || n_q > SPECEXIT_MAX_NQ) return fail(SPECEXIT_EINVAL, "%s: n_q %d outside 1..64", who, n_q);
  if (n_q_heads < 1 || n_q_heads % kv->n_kv_heads) return fail(SPECEXIT_EINVAL, "%s: n_q_heads %d is not a multiple of n_kv_heads %d", who, n_q_heads, kv->n_kv_heads);
  if ((n_q_heads / kv->n_kv_heads) * n_q > 128) return fail(SPECEXIT_EUNSUPPORTED, "%s: more than 128 query rows per KV head", who);
  if (B > 1024) return fail(SPECEXIT_EUNSUPPORTED, "%s: more than 1024 sequences in one call", who);
  memset(&a, 0, sizeof(a));
  a.dtype = kv->dtype;
  a.paged = kv->layout == SPECEXIT_KV_PAGED;
  a.k = kv->k;
  a.v = kv->v;
  a.page_table = kv->page_table;
  a.page_size = a.paged ? kv->page_size : 16;
  a.max_pages = kv->max_pages_per_seq;
  a.l_max = a.paged ? static_cast<int64_t>(kv->max_pages_per_seq) * kv->page_size : kv->l_max;
  a.B = B;
  a.n_q = n_q;
  a.n_blk = n_q;
  a.mask_stride = n_q;
  a.Hq = n_q_heads;
  a.Hkv = kv->n_kv_heads;
  a.d = kv->head_dim;
  a.n_pages = a.paged ? kv->n_pages : 0;
  if (a.l_max < n_q) return fail(SPECEXIT_EINVAL, "%s: the cache holds %lld entries per sequence, fewer than the block's %d", who, static_cast<long long>(a.l_max), n_q);
  if (!attn_plan(a, num_cus())) return fail(SPECEXIT_EUNSUPPORTED, "%s: %d sequences x %d KV heads x %lld cache entries is more than one call can split", who, B, a.Hkv, static_cast<long long>(a.l_max));
  return SPECEXIT_OK;
}

// --------------------------------------------------------------------------- draft plan
struct DraftPlan {
  DraftDims dm;
  bool mfma;
  int B;        // rows of the step: sequences x rows per sequence
  int nseq, W;  // sequences, rows (tree nodes of one level) per sequence
  int top_b;    // continuations reported per row
  int Kmax;
  GemmArgs fc, qkv, o, gu, down, head;
  bool gemv;         // few rows: the layer's projections run as row-streaming GEMVs
  GemvArgs vfc, vqkv, vo, vgu, vdown, vhead;
  AttnArgs attn;
  size_t partial_bytes;
  int ntiles_head;
};

void plan_gemm(GemmArgs& g, int N, int K, int M, int planes, bool mfma, int V) {
  memset(&g, 0, sizeof(g));
  g.N = N;
  g.K = K;
  g.M = M;
  g.planes = mfma ? planes : 1;
  g.V = V;
  g.nseg = 1;
  g.seg_end[0] = g.seg_end[1] = g.seg_end[2] = N;
  choose_ksplit(g, mfma, num_cus());
}

size_t partial_bytes_of(const GemmArgs& g, bool mfma) {
  if (g.V >= 0 && mfma) return 0;
  return static_cast<size_t>(g.ksplit) * g.M * g.planes * g.N * sizeof(float);
}

int32_t make_draft_plan(DraftPlan& p, const specexit_model_desc* d, const specexit_kv_view* kv, int32_t nseq,
                        int32_t W = 1, int32_t top_b = 1) {
  const int32_t B = nseq * W;
  if (!d || d->struct_size != sizeof(specexit_model_desc)) return fail(SPECEXIT_EINVAL, "draft_step: model desc missing or of another ABI size");
  if (!dtype_ok(d->dtype)) return fail(SPECEXIT_EINVAL, "draft_step: unknown dtype %d", d->dtype);
  if (nseq < 1 || W < 1 || B > 64) return fail(SPECEXIT_EINVAL, "draft_step: %d sequences x %d rows outside 1..64 rows", nseq, W);
  if (top_b < 1 || top_b > SPECEXIT_MAX_TOP_B) return fail(SPECEXIT_EINVAL, "draft_step: top_b %d outside 1..%d", top_b, SPECEXIT_MAX_TOP_B);
  if (d->hidden < 64 || d->hidden % 64 || d->hidden > 8192) return fail(SPECEXIT_EUNSUPPORTED, "draft_step: hidden %d must be a multiple of 64 up to 8192", d->hidden);
  if (d->intermediate < 64 || d->intermediate % 64) return fail(SPECEXIT_EUNSUPPORTED, "draft_step: intermediate %d must be a multiple of 64", d->intermediate);
  if (d->vocab < 1) return fail(SPECEXIT_EINVAL, "draft_step: vocab < 1");
  if (d->vocab < top_b) return fail(SPECEXIT_EINVAL, "draft_step: top_b %d exceeds the vocabulary (%d)", top_b, d->vocab);
  if (d->rem_activation < 0 || d->rem_activation > 2) return fail(SPECEXIT_EINVAL, "draft_step: rem_activation %d", d->rem_activation);
  int32_t rc = fill_attn(p.attn, kv, nseq, W, d->n_q_heads, "draft_step");
  if (rc) return rc;
  if (kv->dtype != d->dtype || kv->n_kv_heads != d->n_kv_heads || kv->head_dim != d->head_dim)
    return fail(SPECEXIT_EINVAL, "draft_step: draft kv view does not match the model desc");
  DraftDims& dm = p.dm;
  dm.dtype = d->dtype; dm.D = d->hidden; dm.Hq = d->n_q_heads; dm.Hkv = d->n_kv_heads; dm.d = d->head_dim;
  dm.I = d->intermediate; dm.V = d->vocab; dm.rms_eps = d->rms_eps; dm.rope_theta = d->rope_theta;
  dm.rem_activation = d->rem_activation;
  p.B = B;
  p.nseq = nseq;
  p.W = W;
  p.top_b = top_b;
  const int D = dm.D, Hd = dm.Hq * dm.d, I = dm.I;
  p.Kmax = 2 * D > Hd ? 2 * D : Hd;
  if (I > p.Kmax) p.Kmax = I;
  p.mfma = dm.dtype == SPECEXIT_BF16 && gemm_mfma_supported(B, 2, 2 * D) && gemm_mfma_supported(B, 2, D) &&
           gemm_mfma_supported(B, 2, Hd) && gemm_mfma_supported(B, 2, I);
  plan_gemm(p.fc, D, 2 * D, B, 1, p.mfma, -1);
  plan_gemm(p.qkv, (dm.Hq + 2 * dm.Hkv) * dm.d, D, B, 2, p.mfma, -1);
  p.qkv.nseg = 3;
  p.qkv.seg_end[0] = Hd;
  p.qkv.seg_end[1] = Hd + dm.Hkv * dm.d;
  p.qkv.seg_end[2] = Hd + 2 * dm.Hkv * dm.d;
  plan_gemm(p.o, D, Hd, B, 1, p.mfma, -1);
  plan_gemm(p.gu, 2 * I, D, B, 2, p.mfma, -1);
  p.gu.nseg = 2;
  p.gu.seg_end[0] = I;
  p.gu.seg_end[1] = p.gu.seg_end[2] = 2 * I;
  plan_gemm(p.down, D, I, B, 2, p.mfma, -1);
  p.gemv = p.mfma && gemv_supported(B, D, 2 * D) && gemv_supported(B, (dm.Hq + 2 * dm.Hkv) * dm.d, D) &&
           gemv_supported(B, D, Hd) && gemv_supported(B, 2 * I, D) && gemv_supported(B, D, I) && (dm.d % 2) == 0;
  if (p.gemv) {
    auto plan_v = [&](GemvArgs& g, int N, int K) {
      memset(&g, 0, sizeof(g));
      g.N = N; g.K = K; g.M = B; g.nseg = 1;
      g.seg_end[0] = g.seg_end[1] = g.seg_end[2] = N;
      gemv_plan(g, num_cus());
    };
    plan_v(p.vfc, D, 2 * D);
    plan_v(p.vqkv, (dm.Hq + 2 * dm.Hkv) * dm.d, D);
    p.vqkv.nseg = 3;
    p.vqkv.seg_end[0] = Hd;
    p.vqkv.seg_end[1] = Hd + dm.Hkv * dm.d;
    p.vqkv.seg_end[2] = Hd + 2 * dm.Hkv * dm.d;
    plan_v(p.vo, D, Hd);
    plan_v(p.vgu, 2 * I, D);
    p.vgu.nseg = 2;
    p.vgu.seg_end[0] = I;
    p.vgu.seg_end[1] = p.vgu.seg_end[2] = 2 * I;
    plan_v(p.vdown, D, I);
    plan_v(p.vhead, dm.V + 3, D);
    gemv_plan(p.vhead, num_cus(), 2);   // the long stream does best with two workgroups per compute unit
    // a layer that fits the 256 MB last-level cache is read with ordinary loads, so that part of
    // it is still there one draft step later; a larger one is streamed past the caches
    const size_t layer_bytes = 2 * (static_cast<size_t>(D) * 2 * D + static_cast<size_t>((dm.Hq + 2 * dm.Hkv) * dm.d) * D +
                                    static_cast<size_t>(D) * Hd + static_cast<size_t>(3) * I * D);
    const int stream = layer_bytes > (static_cast<size_t>(240) << 20) ? 1 : 0;
    p.vfc.stream = p.vqkv.stream = p.vo.stream = p.vgu.stream = p.vdown.stream = stream;
    p.vhead.stream = 1;
  }
  plan_gemm(p.head, dm.V + 3, D, B, 2, p.mfma, dm.V);
  p.head.n_extra = 3;
  p.head.top_b = top_b;
  p.ntiles_head = gemm_ntiles(dm.V + 3);
  size_t pb = 0;
  const GemmArgs* all[6] = {&p.fc, &p.qkv, &p.o, &p.gu, &p.down, &p.head};
  for (const GemmArgs* g : all) {
    const size_t b = partial_bytes_of(*g, p.mfma);
    if (b > pb) pb = b;
  }
  p.partial_bytes = pb;
  return SPECEXIT_OK;
}

struct DraftBufs {
  float* act;
  float* partial;
  float* partial2;   // the down projection's partial sums (its input lives in `partial`)
  float *x_buf, *a_buf;
  void *q_buf, *attn_out;
  void* attn_ws;
  float* part_val;
  int* part_idx;
  int32_t* head_am;
  float* extra;
  float* ssq;        // [3][rows][groups of D]: pieces of the sums of squares behind the three norms
  int* counters;     // arrival counters of the reducing GEMM epilogues
  int n_counters;
  size_t total;
};

DraftBufs carve_draft(const DraftPlan& p, void* ws) {
  Carver c(ws);
  DraftBufs b;
  const size_t es = esize(p.dm.dtype);
  b.act = c.take<float>(sizeof(float) * p.B * p.Kmax);
  b.partial = c.take<float>(p.partial_bytes);
  b.partial2 = c.take<float>(p.mfma ? partial_bytes_of(p.down, true) : 0);
  b.x_buf = c.take<float>(sizeof(float) * p.B * p.dm.D);
  b.a_buf = c.take<float>(sizeof(float) * p.B * p.dm.D);
  b.q_buf = c.take<char>(es * p.B * p.dm.Hq * p.dm.d);
  b.attn_out = c.take<char>(es * p.B * p.dm.Hq * p.dm.d);
  b.attn_ws = c.take<char>(attn_workspace_bytes(p.attn));
  b.part_val = c.take<float>(sizeof(float) * p.B * p.ntiles_head * p.top_b);
  b.part_idx = c.take<int>(sizeof(int) * p.B * p.ntiles_head * p.top_b);
  b.head_am = c.take<int32_t>(sizeof(int32_t) * p.B);
  b.extra = c.take<float>(sizeof(float) * p.B * 3);
  const int gd = p.gemv ? 3 * num_cus() : gemm_groups(p.dm.D);   // pieces per row: GEMV workgroups or 128-row groups
  b.ssq = c.take<float>(sizeof(float) * 3 * p.B * gd);
  b.n_counters = 3 * gd + gemm_groups((p.dm.Hq + 2 * p.dm.Hkv) * p.dm.d);
  b.counters = c.take<int>(sizeof(int) * b.n_counters);
  b.total = c.off;
  return b;
}

int32_t run_gemm(GemmArgs g, bool mfma, bool bf16, const void* w0, const void* w1, const void* w2,
                 const DraftBufs& b, hipStream_t s, const char* what) {
  g.w[0] = w0; g.w[1] = w1; g.w[2] = w2;
  g.act = b.act;
  if (g.a_mode == 0) g.a_src = b.act;
  g.partial = b.partial;
  g.part_val = b.part_val;
  g.part_idx = b.part_idx;
  g.extra_out = b.extra;
  return check_hip(mfma ? launch_gemm_mfma(g, s) : launch_gemm_valu(g, bf16, s), what);
}

// Inputs and outputs of one draft forward over p.B = nseq * W rows (row r = sequence r / W).
struct DraftIO {
  const int32_t* tok;        // [rows]
  const void* hidden_in;     // [rows, D]
  const int32_t* pos;        // [nseq] cache entries before this step's block
  int level;                 // rotary position = pos + level
  const int32_t* node;       // [W] cache entry = pos + node (null: pos itself)
  const uint64_t* mask;      // [W] visible block entries per row, shared by the sequences (null: chain)
  int n_blk;                 // block entries that exist after the context
  void* hidden_out;          // [rows, D]
  int32_t* cand_tok;         // [rows, top_b]
  float* cand_logit;         // [rows, top_b] or null
  float *sig_raw, *sig;      // [rows, 3]
  uint32_t flags;
};

int32_t run_draft(DraftPlan& p, const specexit_draft_weights* w, const specexit_kv_view* draft_kv, const DraftIO& io,
                  void* workspace, size_t workspace_bytes, hipStream_t s) {
  int32_t rc;
  const int B = p.B;   // rows
  if (!w || w->struct_size != sizeof(specexit_draft_weights)) return fail(SPECEXIT_EINVAL, "draft_step: weights missing or of another ABI size");
  const void* ptrs[] = {w->embed, w->w_fc, w->ln_attn, w->ln_mlp, w->ln_final, w->w_q, w->w_k, w->w_v,
                        w->w_o, w->w_gate, w->w_up, w->w_down, w->w_head, io.tok, io.hidden_in, io.pos, io.hidden_out,
                        io.cand_tok, io.sig_raw, io.sig};
  for (const void* q : ptrs)
    if (!q) return fail(SPECEXIT_EINVAL, "draft_step: a required pointer is null");
  if (io.hidden_in == io.hidden_out) return fail(SPECEXIT_EINVAL, "draft_step: hidden_in and hidden_out alias");
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return fail(SPECEXIT_EWORKSPACE, "draft_step: workspace null or not 256-byte aligned");
  const DraftBufs b = carve_draft(p, workspace);
  if (workspace_bytes < b.total) return fail(SPECEXIT_EWORKSPACE, "draft_step: workspace %zu < %zu bytes", workspace_bytes, b.total);
  const DraftDims& dm = p.dm;
  const bool bf16 = dm.dtype == SPECEXIT_BF16;
  const bool mf = p.mfma;
  int* const status = status_for(io.flags);

  const int gd = gemm_groups(dm.D);
  g_prof_hook(SPECEXIT_PROF_DRAFT_PROJ_IN, 0, s);
  if (p.gemv) {
    // Few rows: every projection is a row-streaming GEMV whose epilogue finishes the job
    // (residual, rotary embedding + cache write, SiLU gate); the RMSNorms are applied while
    // the next projection stages its activations.
    const int piece = 3 * num_cus();
    auto ssq_of = [&](int which) { return b.ssq + static_cast<size_t>(which) * B * piece; };
    auto normed = [&](GemvArgs& g, int which, const GemvArgs& producer, const float* x, const void* gain) {
      g.a_mode = 3; g.a_src = x; g.a_ssq = ssq_of(which); g.a_nssq = producer.grid; g.a_gain = gain; g.a_eps = dm.rms_eps;
    };
    GemvArgs g = p.vfc;                       // x = W_fc [embed[tok] ; hidden_in]
    g.w[0] = w->w_fc; g.a_mode = 2; g.a_src = io.hidden_in; g.a_embed = w->embed; g.a_tok = io.tok;
    g.a_vocab = dm.V; g.status = status;
    g.out_x = b.x_buf; g.out_ssq = ssq_of(0);
    if ((rc = check_hip(launch_gemv(g, s), "gemv fc"))) return rc;
    g = p.vqkv;                               // q, k, v with rotary embedding, cache write
    g.w[0] = w->w_q; g.w[1] = w->w_k; g.w[2] = w->w_v;
    normed(g, 0, p.vfc, b.x_buf, w->ln_attn);
    g.epi = 1;
    {
      RopeArgs& ra = g.rope;
      ra.pos = io.pos; ra.level = io.level; ra.node = io.node; ra.W = p.W; ra.theta = dm.rope_theta;
      for (int c = 0; c < dm.d / 2; ++c) ra.inv_freq[c] = pow(static_cast<double>(dm.rope_theta), -2.0 * c / dm.d);
      ra.Hq = dm.Hq; ra.Hkv = dm.Hkv; ra.d = dm.d; ra.q_out = b.q_buf; ra.paged = p.attn.paged;
      ra.kc = draft_kv->k; ra.vc = draft_kv->v; ra.page_table = draft_kv->page_table;
      ra.page_size = p.attn.page_size; ra.max_pages = p.attn.max_pages; ra.l_max = p.attn.l_max;
      ra.n_pages = p.attn.n_pages; ra.status = status;
    }
    if ((rc = check_hip(launch_gemv(g, s), "gemv qkv"))) return rc;
  } else if (mf) {
    // Fused form: each projection back into the hidden size finishes its own split-K sums
    // (+ residual) in the workgroup that arrives last, leaving the rows and the pieces of
    // their sums of squares; the next GEMM applies the RMSNorm while it stages its activations,
    // and the down projection applies the SiLU gate the same way.
    // the counters must start at zero and every kernel leaves them at zero: a caller that keeps
    // a zero-filled workspace to this call (same shapes) may say so and save the clearing launch
    if (!(io.flags & SPECEXIT_FLAG_WORKSPACE_PREPARED))
      if ((rc = check_hip(launch_zero_i32(b.counters, b.n_counters, s), "zero counters"))) return rc;
    auto reducing = [&](GemmArgs& g, int which, const float* residual, float* out_x, void* out_store) {
      g.epi = 1;
      g.counters = b.counters + which * gd;
      g.residual = residual;
      g.out_x = out_x;
      g.out_store = out_store;
      g.out_ssq = b.ssq + static_cast<size_t>(which) * B * gd;
    };
    auto normed = [&](GemmArgs& g, int which, const float* x, const void* gain) {
      g.a_mode = 3;
      g.a_src = x;
      g.a_ssq = b.ssq + static_cast<size_t>(which) * B * gd;
      g.a_nssq = gd;
      g.a_gain = gain;
      g.a_eps = dm.rms_eps;
    };
    // x = W_fc [embed[tok] ; hidden_in]
    p.fc.a_mode = 2;   // the GEMM gathers [embed[tok] ; hidden_in] itself
    p.fc.a_src = io.hidden_in;
    p.fc.a_embed = w->embed;
    p.fc.a_tok = io.tok;
    p.fc.a_vocab = dm.V;
    p.fc.status = status;
    reducing(p.fc, 0, nullptr, b.x_buf, nullptr);
    if ((rc = run_gemm(p.fc, mf, bf16, w->w_fc, nullptr, nullptr, b, s, "gemm fc"))) return rc;
    // q, k, v; rotary; cache write; attention over the draft's own cache
    normed(p.qkv, 0, b.x_buf, w->ln_attn);
    p.qkv.epi = 2;     // finished heads are rotated and stored as q / cache entries by the GEMM itself
    p.qkv.counters = b.counters + 3 * gd;
    RopeArgs& ra = p.qkv.rope;
    ra.pos = io.pos; ra.level = io.level; ra.node = io.node; ra.W = p.W; ra.theta = dm.rope_theta;
    for (int c = 0; c < dm.d / 2; ++c) ra.inv_freq[c] = pow(static_cast<double>(dm.rope_theta), -2.0 * c / dm.d);
    ra.Hq = dm.Hq; ra.Hkv = dm.Hkv; ra.d = dm.d; ra.q_out = b.q_buf; ra.paged = p.attn.paged;
    ra.kc = draft_kv->k; ra.vc = draft_kv->v; ra.page_table = draft_kv->page_table;
    ra.page_size = p.attn.page_size; ra.max_pages = p.attn.max_pages; ra.l_max = p.attn.l_max;
    ra.n_pages = p.attn.n_pages; ra.status = status;
    if ((rc = run_gemm(p.qkv, mf, bf16, w->w_q, w->w_k, w->w_v, b, s, "gemm qkv"))) return rc;
  } else {
    if ((rc = check_hip(launch_embed_concat(dm, B, w->embed, io.tok, io.hidden_in, b.act, s, status), "embed_concat"))) return rc;
    if ((rc = run_gemm(p.fc, mf, bf16, w->w_fc, nullptr, nullptr, b, s, "gemm fc"))) return rc;
    if ((rc = check_hip(launch_reduce_norm(dm, B, dm.D, b.partial, p.fc.ksplit, p.fc.planes, nullptr, w->ln_attn,
                                           b.x_buf, nullptr, b.act, s), "norm attn"))) return rc;
    if ((rc = run_gemm(p.qkv, mf, bf16, w->w_q, w->w_k, w->w_v, b, s, "gemm qkv"))) return rc;
    if ((rc = check_hip(launch_rope_kvwrite(dm, B, p.W, b.partial, p.qkv.ksplit, p.qkv.planes, io.pos, io.level, io.node,
                                            b.q_buf, p.attn.paged, draft_kv->k, draft_kv->v, draft_kv->page_table,
                                            p.attn.page_size, p.attn.max_pages, p.attn.l_max, s, p.attn.n_pages, status), "rope"))) return rc;
  }
  g_prof_hook(SPECEXIT_PROF_DRAFT_PROJ_IN, 1, s);
  AttnArgs at = p.attn;
  at.q = b.q_buf;
  at.ctx_len = io.pos;
  at.mask = io.mask;
  at.mask_stride = 0;
  at.n_blk = io.n_blk;
  at.scale = 1.0f / sqrtf(static_cast<float>(dm.d));
  at.out = b.attn_out;
  at.status = status;
  attn_carve(at, b.attn_ws);
  if ((rc = check_hip(launch_attn(at, s, &g_prof_hook, SPECEXIT_PROF_DRAFT_ATTN), "draft attention"))) return rc;
  g_prof_hook(SPECEXIT_PROF_DRAFT_PROJ_OUT, 0, s);
  if (p.gemv) {
    const int piece = 3 * num_cus();
    auto ssq_of = [&](int which) { return b.ssq + static_cast<size_t>(which) * B * piece; };
    GemvArgs g = p.vo;                        // a = x + W_o attn
    g.w[0] = w->w_o; g.a_mode = 1; g.a_src = b.attn_out;
    g.residual = b.x_buf; g.out_x = b.a_buf; g.out_ssq = ssq_of(1);
    if ((rc = check_hip(launch_gemv(g, s), "gemv o"))) return rc;
    g = p.vgu;                                // silu(W_gate m) * (W_up m), m = RMSNorm(a)
    g.w[0] = w->w_gate; g.w[1] = w->w_up;
    g.a_mode = 3; g.a_src = b.a_buf; g.a_ssq = ssq_of(1); g.a_nssq = p.vo.grid; g.a_gain = w->ln_mlp; g.a_eps = dm.rms_eps;
    g.epi = 2; g.out_x = b.act;
    if ((rc = check_hip(launch_gemv(g, s), "gemv gate/up"))) return rc;
    g = p.vdown;                              // y = a + W_down (...)
    g.w[0] = w->w_down; g.a_mode = 0; g.a_src = b.act;
    g.residual = b.a_buf; g.out_x = b.x_buf; g.out_store = io.hidden_out; g.out_ssq = ssq_of(2);
    if ((rc = check_hip(launch_gemv(g, s), "gemv down"))) return rc;
    p.head.a_mode = 3;
    p.head.a_src = b.x_buf;
    p.head.a_ssq = ssq_of(2);
    p.head.a_nssq = p.vdown.grid;
    p.head.a_gain = w->ln_final;
    p.head.a_eps = dm.rms_eps;
  } else if (mf) {
    // a = x + W_o attn
    p.o.a_mode = 1;    // attention output is read in its storage type
    p.o.a_src = b.attn_out;
    p.o.epi = 1;
    p.o.counters = b.counters + gd;
    p.o.residual = b.x_buf;
    p.o.out_x = b.a_buf;
    p.o.out_ssq = b.ssq + static_cast<size_t>(1) * B * gd;
    if ((rc = run_gemm(p.o, mf, bf16, w->w_o, nullptr, nullptr, b, s, "gemm o"))) return rc;
    // y = a + W_down (silu(W_gate m) * W_up m), m = RMSNorm(a)
    p.gu.a_mode = 3;
    p.gu.a_src = b.a_buf;
    p.gu.a_ssq = p.o.out_ssq;
    p.gu.a_nssq = gd;
    p.gu.a_gain = w->ln_mlp;
    p.gu.a_eps = dm.rms_eps;
    if ((rc = run_gemm(p.gu, mf, bf16, w->w_gate, w->w_up, nullptr, b, s, "gemm gate/up"))) return rc;
    // silu(gate) * up once, as fp32 rows: each of the down projection's workgroups stages a K range
    // of all rows, and forming the product there (from the gate/up partial sums) made every one of
    // them re-read and re-add four times the bytes (measured at 16 rows, I = 25600: 104 -> 60 us)
    if ((rc = check_hip(launch_silu_mul(dm, B, b.partial, p.gu.ksplit, p.gu.planes, b.act, s), "silu"))) return rc;
    p.down.a_mode = 0;
    p.down.a_src = b.act;
    p.down.epi = 1;
    p.down.counters = b.counters + 2 * gd;
    p.down.residual = b.a_buf;
    p.down.out_x = b.x_buf;            // y (x is no longer needed)
    p.down.out_store = io.hidden_out;
    p.down.out_ssq = b.ssq + static_cast<size_t>(2) * B * gd;
    {
      GemmArgs g = p.down;
      g.w[0] = w->w_down;
      g.partial = b.partial2;
      if ((rc = check_hip(launch_gemm_mfma(g, s), "gemm down"))) return rc;
    }
    p.head.a_mode = 3;
    p.head.a_src = b.x_buf;
    p.head.a_ssq = p.down.out_ssq;
    p.head.a_nssq = gd;
    p.head.a_gain = w->ln_final;
    p.head.a_eps = dm.rms_eps;
  } else {
    if ((rc = check_hip(launch_unpack_rows(b.attn_out, bf16, B, dm.Hq * dm.d, b.act, s), "unpack attn"))) return rc;
    if ((rc = run_gemm(p.o, mf, bf16, w->w_o, nullptr, nullptr, b, s, "gemm o"))) return rc;
    if ((rc = check_hip(launch_reduce_norm(dm, B, dm.D, b.partial, p.o.ksplit, p.o.planes, b.x_buf, w->ln_mlp,
                                           b.a_buf, nullptr, b.act, s), "norm mlp"))) return rc;
    if ((rc = run_gemm(p.gu, mf, bf16, w->w_gate, w->w_up, nullptr, b, s, "gemm gate/up"))) return rc;
    if ((rc = check_hip(launch_silu_mul(dm, B, b.partial, p.gu.ksplit, p.gu.planes, b.act, s), "silu"))) return rc;
    if ((rc = run_gemm(p.down, mf, bf16, w->w_down, nullptr, nullptr, b, s, "gemm down"))) return rc;
    if ((rc = check_hip(launch_reduce_norm(dm, B, dm.D, b.partial, p.down.ksplit, p.down.planes, b.a_buf, w->ln_final,
                                           nullptr, io.hidden_out, b.act, s), "norm final"))) return rc;
  }
  g_prof_hook(SPECEXIT_PROF_DRAFT_PROJ_OUT, 1, s);
  // widened head (Eq. 1): argmax (or the top_b best) over the vocabulary rows, three signal rows on the side
  if (p.gemv && p.top_b == 1 && !io.cand_logit) {
    // few rows, argmax only: the head is a row stream like the other projections
    GemvArgs g = p.vhead;
    g.w[0] = w->w_head;
    g.a_mode = 3; g.a_src = p.head.a_src; g.a_ssq = p.head.a_ssq; g.a_nssq = p.head.a_nssq; g.a_gain = w->ln_final;
    g.a_eps = dm.rms_eps;
    g.epi = 3; g.V = dm.V; g.n_extra = 3; g.part_val = b.part_val; g.part_idx = b.part_idx; g.extra_out = b.extra;
    {
      ProfScope prof(SPECEXIT_PROF_DRAFT_HEAD_GEMM, s);
      if ((rc = check_hip(launch_gemv(g, s), "gemv head"))) return rc;
    }
    return check_hip(launch_argmax_finalize(b.part_val, b.part_idx, g.grid, B, io.cand_tok, nullptr, s, b.extra,
                                            dm.rem_activation, io.sig_raw, io.sig), "argmax finalize");
  }
  {
    ProfScope prof(SPECEXIT_PROF_DRAFT_HEAD_GEMM, s);
    if ((rc = run_gemm(p.head, mf, bf16, w->w_head, nullptr, nullptr, b, s, "gemm head"))) return rc;
  }
  if (mf) {
    if (p.top_b == 1 && !io.cand_logit)
      return check_hip(launch_argmax_finalize(b.part_val, b.part_idx, p.ntiles_head, B, io.cand_tok, nullptr, s, b.extra,
                                              dm.rem_activation, io.sig_raw, io.sig), "argmax finalize");
    // ranked candidates arrive merged per 128-row workgroup, a plain maximum per 16-row tile
    const int C = (p.top_b > 1 ? gemm_groups(dm.V + 3) : p.ntiles_head) * p.top_b;
    return check_hip(launch_topb_finalize(b.part_val, b.part_idx, C, C, p.top_b, B, io.cand_tok, io.cand_logit, s,
                                          b.extra, dm.rem_activation, io.sig_raw, io.sig), "top-b finalize");
  }
  if ((rc = check_hip(launch_argmax_rows(b.partial, B, dm.V + 3, dm.V, 3, b.head_am, nullptr, b.extra, nullptr, s), "argmax rows"))) return rc;
  if (p.top_b == 1 && !io.cand_logit)
    return check_hip(launch_head_finalize(dm, B, b.head_am, b.extra, io.cand_tok, io.sig_raw, io.sig, s), "head finalize");
  return check_hip(launch_topb_finalize(b.partial, nullptr, dm.V, dm.V + 3, p.top_b, B, io.cand_tok, io.cand_logit, s,
                                        b.extra, dm.rem_activation, io.sig_raw, io.sig), "top-b rows");
}

}  // namespace

extern "C" {

const char* specexit_last_error(void) { return g_err; }

int32_t specexit_copy_probe(const void* src, void* dst, size_t bytes, int32_t nontemporal, void* stream) {
  if (!src || !dst || bytes < 16 || (bytes & 15)) return fail(SPECEXIT_EINVAL, "copy_probe: null pointer or size not a multiple of 16");
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return fail(SPECEXIT_EINVAL, "copy_probe: pointers must be 16-byte aligned");
  return check_hip(launch_copy_probe(src, dst, bytes, nontemporal != 0, static_cast<hipStream_t>(stream)), "copy_probe");
}

int32_t specexit_profile_events(int32_t kernel, void* const* start_events, void* const* stop_events, int32_t n) {
  if (kernel < 0 || kernel >= SPECEXIT_PROF_COUNT) return fail(SPECEXIT_EINVAL, "profile_events: unknown kernel id %d", kernel);
  std::lock_guard<std::mutex> lock(g_prof_mu);
  ProfSlot& sl = g_prof[kernel];
  if (n < 0) return static_cast<int32_t>(sl.used);
  sl.start.clear();
  sl.stop.clear();
  sl.used = 0;
  if (n > 0 && (!start_events || !stop_events)) return fail(SPECEXIT_EINVAL, "profile_events: event arrays are null");
  for (int32_t i = 0; i < n; ++i) {
    sl.start.push_back(static_cast<hipEvent_t>(start_events[i]));
    sl.stop.push_back(static_cast<hipEvent_t>(stop_events[i]));
  }
  return SPECEXIT_OK;
}
uint32_t specexit_version(void) { return 0x00020000u; }

int32_t specexit_set_dev_status(int32_t* dev_status) {
  g_dev_status = dev_status;
  return SPECEXIT_OK;
}

size_t specexit_workspace_bytes(int32_t op, const void* desc, int32_t B, int32_t n_q) {
  switch (op) {
    case SPECEXIT_OP_DRAFT_STEP: {
      const specexit_draft_query* q = static_cast<const specexit_draft_query*>(desc);
      if (!q || q->struct_size != sizeof(*q)) return 0;
      (void)n_q;
      return specexit_draft_step_workspace_bytes(q->desc, q->draft_kv, B);
    }
    case SPECEXIT_OP_DRAFT_TREE_LEVEL: {
      const specexit_draft_query* q = static_cast<const specexit_draft_query*>(desc);
      if (!q || q->struct_size != sizeof(*q)) return 0;
      return specexit_draft_tree_level_workspace_bytes(q->desc, q->draft_kv, B, n_q, q->top_b);
    }
    case SPECEXIT_OP_VERIFY_ATTN: {
      const specexit_attn_query* q = static_cast<const specexit_attn_query*>(desc);
      if (!q || q->struct_size != sizeof(*q)) return 0;
      return specexit_verify_attn_workspace_bytes(q->kv, B, n_q, q->n_q_heads);
    }
    case SPECEXIT_OP_LMHEAD_ARGMAX: {
      const specexit_lmhead_query* q = static_cast<const specexit_lmhead_query*>(desc);
      if (!q || q->struct_size != sizeof(*q) || B < 1 || n_q < 1) return 0;
      return specexit_lmhead_argmax_workspace_bytes(q->dtype, B * n_q, q->hidden, q->vocab, q->n_extra);
    }
    case SPECEXIT_OP_ACCEPT_EXIT:
    case SPECEXIT_OP_KV_COMPACT:
      return 0;   // these calls use no scratch memory
    default:
      fail(SPECEXIT_EINVAL, "workspace_bytes: unknown op %d", op);
      return 0;
  }
}

size_t specexit_draft_step_workspace_bytes(const specexit_model_desc* desc, const specexit_kv_view* draft_kv, int32_t B) {
  DraftPlan p;
  if (make_draft_plan(p, desc, draft_kv, B)) return 0;
  return carve_draft(p, nullptr).total;
}

int32_t specexit_draft_step(const specexit_model_desc* desc, const specexit_draft_weights* w,
                            const specexit_kv_view* draft_kv, int32_t B, const int32_t* tok,
                            const void* hidden_in, const int32_t* pos, void* hidden_out, int32_t* next_tok,
                            float* sig_raw, float* sig, void* workspace, size_t workspace_bytes,
                            uint32_t flags, void* stream) {
  DraftPlan p;
  int32_t rc = make_draft_plan(p, desc, draft_kv, B);
  if (rc) return rc;
  DraftIO io;
  memset(&io, 0, sizeof(io));
  io.flags = flags;
  io.tok = tok; io.hidden_in = hidden_in; io.pos = pos; io.n_blk = 1;
  io.hidden_out = hidden_out; io.cand_tok = next_tok; io.sig_raw = sig_raw; io.sig = sig;
  return run_draft(p, w, draft_kv, io, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t specexit_draft_tree_level_workspace_bytes(const specexit_model_desc* desc, const specexit_kv_view* draft_kv,
                                                 int32_t B, int32_t W, int32_t top_b) {
  DraftPlan p;
  if (make_draft_plan(p, desc, draft_kv, B, W, top_b)) return 0;
  return carve_draft(p, nullptr).total;
}

int32_t specexit_draft_tree_level(const specexit_model_desc* desc, const specexit_draft_weights* w,
                                  const specexit_kv_view* draft_kv, int32_t B, int32_t W, const int32_t* tok,
                                  const void* hidden_in, const int32_t* ctx_len, int32_t level,
                                  const int32_t* node, const uint64_t* anc_mask, int32_t n_blk, int32_t top_b,
                                  void* hidden_out, int32_t* cand_tok, float* cand_logit, float* sig_raw,
                                  float* sig, void* workspace, size_t workspace_bytes, uint32_t flags,
                                  void* stream) {
  DraftPlan p;
  int32_t rc = make_draft_plan(p, desc, draft_kv, B, W, top_b);
  if (rc) return rc;
  if (level < 0) return fail(SPECEXIT_EINVAL, "draft_tree_level: level < 0");
  if (n_blk < 1 || n_blk > SPECEXIT_MAX_NQ) return fail(SPECEXIT_EINVAL, "draft_tree_level: n_blk %d outside 1..64", n_blk);
  if (!node || !anc_mask) return fail(SPECEXIT_EINVAL, "draft_tree_level: node ids or ancestor masks missing");
  if (n_blk > p.attn.l_max) return fail(SPECEXIT_EINVAL, "draft_tree_level: the cache holds fewer entries per sequence than the block's %d", n_blk);
  DraftIO io;
  memset(&io, 0, sizeof(io));
  io.tok = tok; io.hidden_in = hidden_in; io.pos = ctx_len; io.level = level; io.node = node;
  io.mask = anc_mask; io.n_blk = n_blk; io.flags = flags;
  io.hidden_out = hidden_out; io.cand_tok = cand_tok; io.cand_logit = cand_logit; io.sig_raw = sig_raw; io.sig = sig;
  return run_draft(p, w, draft_kv, io, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

size_t specexit_verify_attn_workspace_bytes(const specexit_kv_view* kv, int32_t B, int32_t n_q, int32_t n_q_heads) {
  AttnArgs a;
  if (fill_attn(a, kv, B, n_q, n_q_heads, "verify_attn")) return 0;
  return attn_workspace_bytes(a);
}

int32_t specexit_verify_attn(const specexit_kv_view* kv, int32_t B, int32_t n_q, int32_t n_q_heads, const void* q,
                             const int32_t* ctx_len, const uint64_t* mask, float scale, void* out,
                             void* workspace, size_t workspace_bytes, uint32_t flags, void* stream) {
  AttnArgs a;
  int32_t rc = fill_attn(a, kv, B, n_q, n_q_heads, "verify_attn");
  if (rc) return rc;
  if (!q || !ctx_len || !out) return fail(SPECEXIT_EINVAL, "verify_attn: a required pointer is null");
  if (!(scale > 0.f)) return fail(SPECEXIT_EINVAL, "verify_attn: scale must be positive");
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return fail(SPECEXIT_EWORKSPACE, "verify_attn: workspace null or not 256-byte aligned");
  const size_t need = attn_workspace_bytes(a);
  if (workspace_bytes < need) return fail(SPECEXIT_EWORKSPACE, "verify_attn: workspace %zu < %zu bytes", workspace_bytes, need);
  a.q = q;
  a.ctx_len = ctx_len;
  a.mask = mask;
  a.scale = scale;
  a.out = out;
  a.status = status_for(flags);
  attn_carve(a, workspace);
  return check_hip(launch_attn(a, static_cast<hipStream_t>(stream), &g_prof_hook, SPECEXIT_PROF_VERIFY_ATTN), "verify_attn");
}

namespace {
struct HeadPlan {
  bool mfma;
  GemmArgs g;
  int ntiles;
  size_t act_bytes, partial_bytes, pv_bytes, pack_bytes;
};
int32_t make_head_plan(HeadPlan& h, int32_t dtype, int32_t M, int32_t D, int32_t V, int32_t n_extra) {
  if (!dtype_ok(dtype)) return fail(SPECEXIT_EINVAL, "lmhead_argmax: unknown dtype %d", dtype);
  if (M < 1 || M > 144) return fail(SPECEXIT_EINVAL, "lmhead_argmax: M %d outside 1..144", M);
  if (D < 8 || D % 8) return fail(SPECEXIT_EUNSUPPORTED, "lmhead_argmax: D %d must be a multiple of 8", D);
  if (V < 1 || n_extra < 0 || n_extra > 16) return fail(SPECEXIT_EINVAL, "lmhead_argmax: bad V or n_extra");
  h.mfma = dtype == SPECEXIT_BF16 && gemm_mfma_supported(M, 1, D);
  plan_gemm(h.g, V + n_extra, D, M, 1, h.mfma, V);
  h.g.n_extra = n_extra;
  h.ntiles = gemm_ntiles(V + n_extra);
  h.act_bytes = (!h.mfma && dtype == SPECEXIT_BF16) ? sizeof(float) * M * D : 0;
  h.partial_bytes = h.mfma ? 0 : sizeof(float) * M * (static_cast<size_t>(V) + n_extra);
  h.pv_bytes = h.mfma ? sizeof(float) * M * (h.g.wide ? head_wide_groups(h.g) : h.ntiles) : 0;
  h.pack_bytes = h.mfma ? head_wide_pack_bytes(h.g) : 0;
  return SPECEXIT_OK;
}
}  // namespace

size_t specexit_lmhead_argmax_workspace_bytes(int32_t dtype, int32_t M, int32_t D, int32_t V, int32_t n_extra) {
  HeadPlan h;
  if (make_head_plan(h, dtype, M, D, V, n_extra)) return 0;
  size_t t = align256(h.act_bytes) + align256(h.partial_bytes) + 2 * align256(h.pv_bytes) + align256(h.pack_bytes);
  return t ? t : 256;
}

int32_t specexit_lmhead_argmax(int32_t dtype, int32_t M, int32_t D, int32_t V, int32_t n_extra, const void* hidden,
                               const void* w, int32_t* argmax, float* max_logit, float* extra_out,
                               float* logits_dbg, void* workspace, size_t workspace_bytes, uint32_t flags,
                               void* stream) {
  (void)flags;
  HeadPlan h;
  int32_t rc = make_head_plan(h, dtype, M, D, V, n_extra);
  if (rc) return rc;
  if (!hidden || !w || !argmax) return fail(SPECEXIT_EINVAL, "lmhead_argmax: a required pointer is null");
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return fail(SPECEXIT_EWORKSPACE, "lmhead_argmax: workspace null or not 256-byte aligned");
  const size_t need = specexit_lmhead_argmax_workspace_bytes(dtype, M, D, V, n_extra);
  if (workspace_bytes < need) return fail(SPECEXIT_EWORKSPACE, "lmhead_argmax: workspace %zu < %zu bytes", workspace_bytes, need);
  hipStream_t s = static_cast<hipStream_t>(stream);
  Carver c(workspace);
  float* act = c.take<float>(h.act_bytes);
  float* partial = c.take<float>(h.partial_bytes);
  float* pv = c.take<float>(h.pv_bytes);
  int* pi = c.take<int>(h.pv_bytes);
  char* packed = c.take<char>(h.pack_bytes);
  GemmArgs g = h.g;
  g.a_packed = packed;
  g.w[0] = w;
  g.extra_out = n_extra ? extra_out : nullptr;
  g.logits_dbg = logits_dbg;
  const bool bf16 = dtype == SPECEXIT_BF16;
  if (h.mfma) {
    g.a_mode = 1;
    g.a_src = hidden;
    g.part_val = pv;
    g.part_idx = pi;
    {
      ProfScope prof(SPECEXIT_PROF_LMHEAD_GEMM, s);
      if ((rc = check_hip(launch_gemm_mfma(g, s), "gemm lm head"))) return rc;
    }
    return check_hip(launch_argmax_finalize(pv, pi, g.wide ? head_wide_groups(g) : h.ntiles, M, argmax, max_logit, s), "argmax finalize");
  }
  if (bf16) {
    if ((rc = check_hip(launch_unpack_rows(hidden, true, M, D, act, s), "unpack hidden"))) return rc;
    g.act = act;
  } else {
    g.act = static_cast<const float*>(hidden);
  }
  g.partial = partial;
  {
    ProfScope prof(SPECEXIT_PROF_LMHEAD_GEMM, s);
    if ((rc = check_hip(launch_gemm_valu(g, bf16, s), "gemv lm head"))) return rc;
  }
  return check_hip(launch_argmax_rows(partial, M, V + n_extra, V, n_extra, argmax, max_logit,
                                      n_extra ? extra_out : nullptr, logits_dbg, s), "argmax rows");
}

namespace {
// Scratch of specexit_lmhead_argmax_noalloc: one copy per GPU, held until the process ends.
// In host code the array's name is only a stand-in; its device address comes from
// hipGetSymbolAddress, once per device, and that address is what the kernels get.
constexpr size_t kScratchBytes = SPECEXIT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_addr[kMaxDevices] = {};
std::mutex g_scratch_mu;

int32_t scratch_of_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return check_hip(e, "lmhead_argmax_noalloc: hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(SPECEXIT_EUNSUPPORTED, "lmhead_argmax_noalloc: device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_addr[dev]) {
    void* addr = nullptr;
    e = hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !addr) return check_hip(e == hipSuccess ? hipErrorInvalidSymbol : e, "lmhead_argmax_noalloc: address of the built-in scratch buffer");
    g_scratch_addr[dev] = addr;
  }
  *out = g_scratch_addr[dev];
  return SPECEXIT_OK;
}
}  // namespace

int32_t specexit_lmhead_argmax_noalloc(int32_t dtype, int32_t M, int32_t D, int32_t V, int32_t n_extra,
                                       const void* hidden, const void* w, int32_t* argmax, float* max_logit,
                                       float* extra_out, float* logits_dbg, uint32_t flags, void* stream) {
  HeadPlan h;
  int32_t rc = make_head_plan(h, dtype, M, D, V, n_extra);
  if (rc) return rc;
  const size_t need = specexit_lmhead_argmax_workspace_bytes(dtype, M, D, V, n_extra);
  if (need > kScratchBytes)
    return fail(SPECEXIT_EWORKSPACE, "lmhead_argmax_noalloc: this shape needs %zu bytes of scratch, the built-in buffer holds %zu "
                "(use specexit_lmhead_argmax with a workspace of the caller's)", need, kScratchBytes);
  void* addr = nullptr;
  if ((rc = scratch_of_current_device(&addr))) return rc;
  // every word of the scratch a call reads was written by that same call's kernels (argmax candidates,
  // the activations in operand order, or the logits of the ALU path): nothing has to start at zero
  return specexit_lmhead_argmax(dtype, M, D, V, n_extra, hidden, w, argmax, max_logit, extra_out, logits_dbg, addr,
                                kScratchBytes, flags, stream);
}

int32_t specexit_accept_exit(const specexit_exit_cfg* cfg, int32_t B, int32_t n_q, const int32_t* block_tok,
                             const int32_t* parent, const int32_t* target_argmax, const float* sig,
                             const int32_t* ctx_len, const int32_t* split_tok, int32_t S, float* ewma,
                             int32_t* n_obs, int32_t* is_thinking, float* smooth_state, int32_t* accept_len,
                             int32_t* accept_path,
                             int32_t* recover_tok, int32_t* last_node, int32_t* exit_flag, int32_t* new_ctx_len,
                             uint32_t flags, void* stream) {
  (void)flags;
  if (!cfg || cfg->struct_size != sizeof(specexit_exit_cfg)) return fail(SPECEXIT_EINVAL, "accept_exit: cfg missing or of another ABI size");
  if (B < 1) return fail(SPECEXIT_EINVAL, "accept_exit: B < 1");
  if (n_q < 1 || n_q > SPECEXIT_MAX_NQ) return fail(SPECEXIT_EINVAL, "accept_exit: n_q %d outside 1..64", n_q);
  if (S < 0 || (S > 0 && !split_tok)) return fail(SPECEXIT_EINVAL, "accept_exit: split token set missing");
  if (!(cfg->alpha >= 0.f && cfg->alpha <= 1.f)) return fail(SPECEXIT_EINVAL, "accept_exit: alpha outside [0,1]");
  if (cfg->smoother < SPECEXIT_SMOOTH_EWMA || cfg->smoother > SPECEXIT_SMOOTH_PARAGRAPH)
    return fail(SPECEXIT_EUNSUPPORTED, "accept_exit: smoother %d", cfg->smoother);
  if (cfg->window < 0 || cfg->window > 16) return fail(SPECEXIT_EINVAL, "accept_exit: window %d outside 1..16 (0 = 10)", cfg->window);
  if (cfg->smoother >= SPECEXIT_SMOOTH_WINDOW && !smooth_state)
    return fail(SPECEXIT_EINVAL, "accept_exit: smoother %d needs smooth_state", cfg->smoother);
  static_assert(kSmoothWords == SPECEXIT_SMOOTH_WORDS, "history size of the ABI and of the kernel differ");
  const void* ptrs[] = {block_tok, target_argmax, sig, ctx_len, ewma, n_obs, is_thinking, accept_len,
                        accept_path, recover_tok, last_node, exit_flag, new_ctx_len};
  for (const void* q : ptrs)
    if (!q) return fail(SPECEXIT_EINVAL, "accept_exit: a required pointer is null");
  ExitArgs a;
  a.alpha = cfg->alpha; a.thr_conf = cfg->thr_conf; a.thr_prog = cfg->thr_prog; a.thr_rem = cfg->thr_rem;
  a.signal_mask = cfg->signal_mask; a.smoother = cfg->smoother; a.split_pick = cfg->split_pick;
  a.window = cfg->window ? cfg->window : 10; a.smooth_state = smooth_state;
  a.check_root = cfg->check_root; a.stop_think_token = cfg->stop_think_token;
  a.B = B; a.n_q = n_q; a.S = S;
  a.block_tok = block_tok; a.parent = parent; a.target_argmax = target_argmax; a.sig = sig;
  a.ctx_len = ctx_len; a.split_tok = split_tok; a.ewma = ewma; a.n_obs = n_obs; a.is_thinking = is_thinking;
  a.accept_len = accept_len; a.accept_path = accept_path; a.recover_tok = recover_tok; a.last_node = last_node;
  a.exit_flag = exit_flag; a.new_ctx_len = new_ctx_len;
  return check_hip(launch_accept_exit(a, static_cast<hipStream_t>(stream)), "accept_exit");
}

struct specexit_graph {
  hipGraphExec_t exec;
};

int32_t specexit_graph_begin(void* stream) {
  if (!stream) return fail(SPECEXIT_EINVAL, "graph_begin: the null stream cannot be captured");
  return check_hip(hipStreamBeginCapture(static_cast<hipStream_t>(stream), hipStreamCaptureModeThreadLocal), "graph_begin");
}

int32_t specexit_graph_end(void* stream, specexit_graph** out) {
  if (!stream || !out) return fail(SPECEXIT_EINVAL, "graph_end: null stream or result pointer");
  *out = nullptr;
  hipGraph_t graph = nullptr;
  int32_t rc = check_hip(hipStreamEndCapture(static_cast<hipStream_t>(stream), &graph), "graph_end");
  if (rc) return rc;
  if (!graph) return fail(SPECEXIT_ELAUNCH, "graph_end: the capture produced no graph");
  hipGraphExec_t exec = nullptr;
  rc = check_hip(hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0), "graph instantiate");
  (void)hipGraphDestroy(graph);
  if (rc) return rc;
  specexit_graph* g = new (std::nothrow) specexit_graph;
  if (!g) {
    (void)hipGraphExecDestroy(exec);
    return fail(SPECEXIT_ELAUNCH, "graph_end: out of host memory");
  }
  g->exec = exec;
  *out = g;
  return SPECEXIT_OK;
}

int32_t specexit_graph_launch(const specexit_graph* graph, void* stream) {
  if (!graph) return fail(SPECEXIT_EINVAL, "graph_launch: null graph");
  return check_hip(hipGraphLaunch(graph->exec, static_cast<hipStream_t>(stream)), "graph_launch");
}

int32_t specexit_graph_destroy(specexit_graph* graph) {
  if (!graph) return SPECEXIT_OK;
  const hipError_t e = hipGraphExecDestroy(graph->exec);
  delete graph;
  return check_hip(e, "graph_destroy");
}

int32_t specexit_workspace_prepare(void* workspace, size_t workspace_bytes, void* stream) {
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255)) return fail(SPECEXIT_EWORKSPACE, "workspace_prepare: workspace null or not 256-byte aligned");
  if (workspace_bytes / 4 > 0x7fffffff) return fail(SPECEXIT_EINVAL, "workspace_prepare: workspace too large");
  if (workspace_bytes < 4) return SPECEXIT_OK;
  return check_hip(launch_zero_i32(static_cast<int*>(workspace), static_cast<int>(workspace_bytes / 4),
                                   static_cast<hipStream_t>(stream)), "workspace_prepare");
}

int32_t specexit_tree_gather(int32_t dtype, int32_t B, int32_t W_prev, int32_t top_b, int32_t W_next, int32_t D,
                             int32_t n_q, const int32_t* src_row, const int32_t* rank, const int32_t* node,
                             const int32_t* cand_tok, const void* hidden_prev, int32_t* tok_next,
                             void* hidden_next, int32_t* block_tok, uint32_t flags, void* stream) {
  (void)flags;
  if (!dtype_ok(dtype)) return fail(SPECEXIT_EINVAL, "tree_gather: unknown dtype %d", dtype);
  if (B < 1 || W_prev < 1 || W_next < 1 || B > 65535 || W_next > SPECEXIT_MAX_NQ || W_prev > SPECEXIT_MAX_NQ)
    return fail(SPECEXIT_EINVAL, "tree_gather: B, W_prev or W_next out of range");
  if (top_b < 1 || top_b > SPECEXIT_MAX_TOP_B) return fail(SPECEXIT_EINVAL, "tree_gather: top_b %d outside 1..%d", top_b, SPECEXIT_MAX_TOP_B);
  if (n_q < 1 || n_q > SPECEXIT_MAX_NQ) return fail(SPECEXIT_EINVAL, "tree_gather: n_q %d outside 1..64", n_q);
  if (!src_row || !rank || !node || !cand_tok || !tok_next) return fail(SPECEXIT_EINVAL, "tree_gather: a required pointer is null");
  TreeGatherArgs a;
  memset(&a, 0, sizeof(a));
  a.B = B; a.W_prev = W_prev; a.top_b = top_b; a.W_next = W_next; a.n_q = n_q;
  a.src_row = src_row; a.rank = rank; a.node = node; a.cand_tok = cand_tok; a.tok_next = tok_next;
  a.block_tok = block_tok;
  if (hidden_next) {
    if (!hidden_prev || hidden_prev == hidden_next) return fail(SPECEXIT_EINVAL, "tree_gather: hidden_prev missing or aliasing hidden_next");
    if (D < 1 || (D * esize(dtype)) % 16) return fail(SPECEXIT_EINVAL, "tree_gather: D * element size must be a multiple of 16");
    a.hidden_prev = hidden_prev; a.hidden_next = hidden_next;
    a.row_bytes = static_cast<int>(D * esize(dtype));
  }
  return check_hip(launch_tree_gather(a, static_cast<hipStream_t>(stream)), "tree_gather");
}

int32_t specexit_kv_compact(const specexit_kv_view* kv, int32_t n_layers, int64_t layer_stride_bytes, int32_t B,
                            int32_t n_q, const int32_t* ctx_len, const int32_t* accept_path,
                            const int32_t* accept_len, const int32_t* last_node, const void* block_hidden,
                            int32_t D, void* hidden_next, uint32_t flags, void* stream) {
  int32_t rc = check_kv(kv, "kv_compact");
  if (rc) return rc;
  if (B < 1) return fail(SPECEXIT_EINVAL, "kv_compact: B < 1");
  if (n_q < 1 || n_q > SPECEXIT_MAX_NQ) return fail(SPECEXIT_EINVAL, "kv_compact: n_q %d outside 1..64", n_q);
  if (n_layers < 1) return fail(SPECEXIT_EINVAL, "kv_compact: n_layers < 1");
  if (n_layers > 1 && (layer_stride_bytes <= 0 || layer_stride_bytes % 16))
    return fail(SPECEXIT_EINVAL, "kv_compact: layer stride must be a positive multiple of 16 bytes");
  if (!ctx_len || !accept_path || !accept_len) return fail(SPECEXIT_EINVAL, "kv_compact: a required pointer is null");
  CompactArgs a;
  memset(&a, 0, sizeof(a));
  a.paged = kv->layout == SPECEXIT_KV_PAGED;
  a.k = kv->k; a.v = kv->v; a.page_table = kv->page_table;
  a.page_size = a.paged ? kv->page_size : 16;
  a.max_pages = kv->max_pages_per_seq;
  a.l_max = a.paged ? static_cast<int64_t>(kv->max_pages_per_seq) * kv->page_size : kv->l_max;
  a.n_pages = a.paged ? kv->n_pages : 0;
  a.status = status_for(flags);
  a.layer_stride_bytes = n_layers > 1 ? layer_stride_bytes : 0;
  a.n_layers = n_layers; a.B = B; a.n_q = n_q; a.Hkv = kv->n_kv_heads;
  a.row_bytes = static_cast<int>(kv->head_dim * esize(kv->dtype));
  a.ctx_len = ctx_len; a.accept_path = accept_path; a.accept_len = accept_len; a.last_node = last_node;
  if (block_hidden) {
    if (!last_node || !hidden_next) return fail(SPECEXIT_EINVAL, "kv_compact: block_hidden given without last_node / hidden_next");
    if (D < 1 || (D * esize(kv->dtype)) % 16) return fail(SPECEXIT_EINVAL, "kv_compact: D * element size must be a multiple of 16");
    a.block_hidden = block_hidden; a.hidden_next = hidden_next;
    a.hidden_row_bytes = static_cast<int>(D * esize(kv->dtype));
  }
  if (!kv_compact_supported(a)) return fail(SPECEXIT_EUNSUPPORTED, "kv_compact: block of %d nodes with %d-byte rows", n_q, a.row_bytes);
  if (kv->n_kv_heads > 65535 || B > 65535 || n_layers > 65535) return fail(SPECEXIT_EUNSUPPORTED, "kv_compact: grid too large");
  return check_hip(launch_kv_compact(a, static_cast<hipStream_t>(stream)), "kv_compact");
}

}  // extern "C"
