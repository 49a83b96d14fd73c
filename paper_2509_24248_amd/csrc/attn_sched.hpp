// Work split of the split-KV attention kernels.
//
// The context lengths live on the device, so the host cannot cut the caches into equal pieces.
// The kernels do it themselves: the keys of every (sequence, KV head) unit are counted in
// granules of 64, the units are laid end to end on one line of T granules (unit u = b * Hkv + g
// starts at Hkv * S[b] + g * n_b, S = prefix sums of the sequences' granule counts n_b), and
// workgroup w of W takes the granules [w T / W, (w + 1) T / W).  Every workgroup therefore has
// the same amount of cache to read whatever the mix of lengths, all of them are resident at
// once, and nobody waits for a long sequence's last chunk.  A workgroup whose range crosses a
// unit boundary finishes one unit's partial result and starts the next (a "segment" per unit).
// Segment (w, u) writes partial slot w + u: both grow along the line, so the slots of one unit
// are consecutive and no two segments share one; W + units slots are enough.
#pragma once
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

constexpr int kAttnGran = 64;        // keys per granule
constexpr int kAttnMaxSeqs = 1024;   // sequences per launch (prefix table in LDS)

// A context length as the kernels use it: forced into 0 .. l_max - n_blk so that no access can
// leave the cache whatever the array holds.
__device__ __forceinline__ int attn_ctx_len(const AttnArgs& a, int b) {
  const int raw = a.ctx_len[b];
  const int hi = static_cast<int>(a.l_max) - a.n_blk;
  const int L = min(max(raw, 0), hi);
  if (L != raw) report_status(a.status, kStatusBadLength);
  return L;
}

// Prefix sums S[0 .. B] of the sequences' granule counts, built by the first wave; every thread
// of the workgroup calls this, and the table is ready when it returns.
__device__ __forceinline__ void attn_sched_build(const AttnArgs& a, int* S) {
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    int run = 0;
    for (int c = 0; c < a.B; c += 64) {
      const int b = c + lane;
      int x = 0;
      if (b < a.B) x = (attn_ctx_len(a, b) + a.n_blk + kAttnGran - 1) / kAttnGran;
#pragma unroll
      for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o, 64);
        if (lane >= o) x += y;
      }
      if (b < a.B) S[b + 1] = run + x;
      run += __shfl(x, 63, 64);
    }
    if (lane == 0) S[0] = 0;
  }
  __syncthreads();
}

// Workgroups that take part: at least two granules each while there are that many.
__device__ __forceinline__ int attn_sched_workgroups(int T, int wgrid) { return max(1, min(wgrid, T >> 1)); }

__device__ __forceinline__ int attn_sched_lo(int w, int T, int W) {
  return static_cast<int>(static_cast<int64_t>(w) * T / W);
}

// first and last workgroup whose range holds a granule of [p, p + n)
__device__ __forceinline__ int attn_sched_owner(int p, int T, int W) {
  return static_cast<int>((static_cast<int64_t>(p + 1) * W - 1) / T);
}

struct AttnSeg {
  int b, g;      // unit
  int s0, s1;    // keys [s0, s1) of the unit
  int L;         // context length of the sequence (block entries follow)
  int next;      // granule on the line where the next segment starts
};

// The segment that starts at granule x of the line and ends at the unit's end or at `hi`.
// Uniform over the workgroup; S in LDS.
__device__ __forceinline__ AttnSeg attn_sched_segment(const AttnArgs& a, const int* S, int x, int hi) {
  const int lane = threadIdx.x & 63;
  int b = 0;
  for (int c = 0; c < a.B; c += 64) {
    const int i = c + lane;
    const bool before = i < a.B && static_cast<int64_t>(a.Hkv) * S[i + 1] <= x;
    b += __popcll(__builtin_amdgcn_ballot_w64(before));
  }
  b = __builtin_amdgcn_readfirstlane(min(b, a.B - 1));
  const int n = S[b + 1] - S[b];
  const int rel = x - a.Hkv * S[b];
  AttnSeg s;
  s.b = b;
  s.g = min(rel / n, a.Hkv - 1);
  const int g0 = min(rel - s.g * n, n - 1);     // first granule inside the unit
  const int g1 = min(n, g0 + (hi - x));
  s.L = attn_ctx_len(a, b);
  s.s0 = g0 * kAttnGran;
  s.s1 = min(s.L + a.n_blk, g1 * kAttnGran);
  s.next = x + max(g1 - g0, 1);                 // (the minima above cannot bind while S is the table of these lengths)
  return s;
}

}  // namespace sx
