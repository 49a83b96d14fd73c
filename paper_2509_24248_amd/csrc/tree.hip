// Between two levels of tree drafting: the nodes of the next level take their tokens from
// their parents' ranked continuations and their input hidden state from their parents'
// output (the block that the target's verification forward later checks, Alg. 1, is filled in on the way).
// A few KB per call: latency-bound, one launch per level.
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

__global__ __launch_bounds__(256) void k_tree_gather(const TreeGatherArgs a) {
  const int wn = blockIdx.x, b = blockIdx.y;
  int src = a.src_row[wn];
  int rk = a.rank[wn];
  const int nd = a.node[wn];
  src = max(0, min(src, a.W_prev - 1));
  rk = max(0, min(rk, a.top_b - 1));
  if (threadIdx.x == 0) {
    const int32_t t = a.cand_tok[(static_cast<size_t>(b) * a.W_prev + src) * a.top_b + rk];
    a.tok_next[static_cast<size_t>(b) * a.W_next + wn] = t;
    if (a.block_tok && nd >= 0 && nd < a.n_q) a.block_tok[static_cast<size_t>(b) * a.n_q + nd] = t;
  }
  if (a.hidden_next) {
    const uint4* s = reinterpret_cast<const uint4*>(static_cast<const char*>(a.hidden_prev) +
                                                    (static_cast<size_t>(b) * a.W_prev + src) * a.row_bytes);
    uint4* d = reinterpret_cast<uint4*>(static_cast<char*>(a.hidden_next) +
                                        (static_cast<size_t>(b) * a.W_next + wn) * a.row_bytes);
    for (int i = threadIdx.x; i < (a.row_bytes >> 4); i += 256) d[i] = s[i];
  }
}

}  // namespace

hipError_t launch_tree_gather(const TreeGatherArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_tree_gather, dim3(a.W_next, a.B), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace sx
