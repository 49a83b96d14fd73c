// Stages 4 and 5 of the round (Alg. 1): greedy acceptance of the draft block against the
// target's argmax tokens, smoothing of the three exit signals (Appendix, EWMA with
// alpha = 0.1, or one of the appendix's other smoothers), the stop thresholds (Appendix, "Stop Threshold") and the step-split gate
// with truncation (Sec. 3.3 "Stopping Conditions").  One thread per sequence: the work is
// a few dozen integer operations, so the kernel costs one launch and nothing else, which
// is the point the paper makes against probing-based exits.
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

__device__ __forceinline__ bool in_sorted(const int32_t* a, int n, int32_t key) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    const int32_t v = a[mid];
    if (v == key) return true;
    if (v < key) lo = mid + 1; else hi = mid;
  }
  return false;
}

__global__ __launch_bounds__(64) void k_accept_exit(const ExitArgs a) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= a.B) return;
  const int n = a.n_q;
  const int32_t* tok = a.block_tok + static_cast<size_t>(b) * n;
  const int32_t* am = a.target_argmax + static_cast<size_t>(b) * n;
  const int32_t* par = a.parent ? a.parent + static_cast<size_t>(b) * n : nullptr;
  int32_t* path = a.accept_path + static_cast<size_t>(b) * n;

  // ---- smoothing (Appendix, "Signal Smoothing"); the first observation seeds x
  //  EWMA       x_t = alpha s_t + (1 - alpha) x_{t-1}
  //  window     mean of the last n = min(N, observations) values, kept in a ring of N
  //  momentum   latest value + mean of the n-1 differences between the last n values; the
  //             differences telescope to (latest - oldest of the ring) / (n - 1)
  //  paragraph  mean of the values since the last paragraph end: a compensated running sum
  //             (words 0, 1 of the signal's row) and a count (word 2 of row 0)
  int thinking = a.is_thinking[b];
  float x[3];
#pragma unroll
  for (int j = 0; j < 3; ++j) x[j] = a.ewma[b * 3 + j];
  float* hist = a.smooth_state ? a.smooth_state + static_cast<size_t>(b) * kSmoothWords : nullptr;
  if (thinking) {
    const int seen = max(a.n_obs[b], 0);   // caller-owned state: a negative count must not reach the ring index
    const int N = a.window;
    const int n = min(seen + 1, N);
    int par_count = 0;
    if (a.smoother == 4) par_count = __float_as_int(hist[2]) + 1;
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const float s = a.sig[b * 3 + j];
      float* h = hist + 16 * j;
      if (a.smoother == 0) {
        x[j] = seen == 0 ? s : __fadd_rn(__fmul_rn(a.alpha, s), __fmul_rn(1.0f - a.alpha, x[j]));
      } else if (a.smoother == 1) {
        x[j] = s;
      } else if (a.smoother == 2 || a.smoother == 3) {
        h[seen % N] = s;
        const float oldest = h[(seen + 1 - n) % N];
        if (a.smoother == 2) {
          float sum = 0.f;
          for (int i = seen + 1 - n; i <= seen; ++i) sum += h[i % N];
          x[j] = sum / static_cast<float>(n);
        } else {
          x[j] = n == 1 ? s : s + (s - oldest) / static_cast<float>(n - 1);
        }
      } else {
        // Kahan step: the mean of a long paragraph keeps full float accuracy
        const float y = s - h[1];
        const float t = __fadd_rn(h[0], y);
        h[1] = __fsub_rn(__fsub_rn(t, h[0]), y);
        h[0] = t;
        x[j] = t / static_cast<float>(par_count);
      }
      a.ewma[b * 3 + j] = x[j];
    }
    if (a.smoother == 4) hist[2] = __int_as_float(par_count);
    a.n_obs[b] = seen + 1;
  }

  // ---- acceptance: follow matching children from the root
  int cur = 0, len = 0;
  while (true) {
    int nxt = -1;
    const int32_t want = am[cur];
    for (int c = cur + 1; c < n; ++c) {
      const int p = par ? par[c] : c - 1;
      if (p == cur && tok[c] == want) { nxt = c; break; }
    }
    if (nxt < 0) break;
    path[len++] = nxt;
    cur = nxt;
  }
  int32_t t_rec = am[cur];

  // ---- exit gate
  bool pass = true;
  if (a.signal_mask & 1u) pass = pass && (x[0] > a.thr_conf);
  if (a.signal_mask & 2u) pass = pass && (x[1] > a.thr_prog);
  if (a.signal_mask & 4u) pass = pass && (x[2] < a.thr_rem);
  int flag = 0;
  if (thinking && (pass || a.smoother == 4)) {
    int cut = -1;  // number of accepted drafts kept when the exit fires
    if (a.check_root && in_sorted(a.split_tok, a.S, tok[0])) cut = 0;
    for (int j = 0; j < len; ++j) {
      if (in_sorted(a.split_tok, a.S, tok[path[j]])) {
        if (a.split_pick == 0) { if (cut < 0) cut = j + 1; }
        else cut = j + 1;
      }
    }
    if (cut >= 0 && !pass) {
      // a step-split token was accepted but the sequence goes on thinking: its paragraph ends
#pragma unroll
      for (int j = 0; j < 3; ++j) { hist[16 * j] = 0.f; hist[16 * j + 1] = 0.f; }
      hist[2] = __int_as_float(0);
    } else if (cut >= 0) {
      len = cut;
      cur = len ? path[len - 1] : 0;
      t_rec = a.stop_think_token;
      thinking = 0;
      flag = 1;
      a.is_thinking[b] = 0;
    }
  }
  for (int j = len; j < n; ++j) path[j] = -1;
  a.accept_len[b] = len;
  a.recover_tok[b] = t_rec;
  a.last_node[b] = cur;
  a.exit_flag[b] = flag;
  a.new_ctx_len[b] = a.ctx_len[b] + 1 + len;
}

}  // namespace

hipError_t launch_accept_exit(const ExitArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_accept_exit, dim3((a.B + 63) / 64), dim3(64), 0, s, a);
  return hipGetLastError();
}

}  // namespace sx
