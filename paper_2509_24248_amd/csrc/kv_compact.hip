// What a round leaves behind for the next one (Alg. 1, the cache-update step inside the exit
// branch, applied after every round): the K/V entries of the accepted path, stored at cache positions
// L + node during verification, move to L + 1 + j so that the cache again holds a plain
// sequence; the target's hidden state of the last accepted node is handed on as the next
// round's first draft input.  A few KB per (sequence, KV head, layer): latency-bound, so one
// launch covers every layer.
//
// grid = (KV heads, sequences, layers).  A workgroup reads every row it has to move into
// registers, meets at a barrier, and only then writes: targets and sources overlap (path
// (2, 3) writes entry 2 while entry 2 is still a source), and no other workgroup touches
// the same (sequence, head, layer).  Chains move nothing (node j + 1 already sits at
// L + 1 + j) and return at once.
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

constexpr int kThreads = 256;
constexpr int kMaxItems = 16;   // 16-byte pieces per thread: 2 * 63 rows * 32 pieces / 256 threads

__global__ __launch_bounds__(kThreads) void k_kv_compact(const CompactArgs a) {
  const int h = blockIdx.x, b = blockIdx.y, layer = blockIdx.z;
  const int L = a.ctx_len[b];
  int m = a.accept_len[b];
  m = max(0, min(m, a.n_q - 1));
  const int32_t* path = a.accept_path + static_cast<size_t>(b) * a.n_q;
  const int lpr = a.row_bytes >> 4;                 // 16-byte pieces per row
  const bool in_cache = L >= 0 && static_cast<int64_t>(L) + a.n_q <= a.l_max;
  if (!in_cache) report_status(a.status, kStatusBadLength);

  // ---- hidden state of the last accepted node -> next round's draft input
  if (h == 0 && layer == 0 && a.block_hidden) {
    int node = a.last_node[b];
    if (node < 0 || node >= a.n_q) report_status(a.status, kStatusBadNode);
    node = max(0, min(node, a.n_q - 1));
    const uint4* src = reinterpret_cast<const uint4*>(static_cast<const char*>(a.block_hidden) +
                                                      (static_cast<size_t>(b) * a.n_q + node) * a.hidden_row_bytes);
    uint4* dst = reinterpret_cast<uint4*>(static_cast<char*>(a.hidden_next) + static_cast<size_t>(b) * a.hidden_row_bytes);
    for (int i = threadIdx.x; i < (a.hidden_row_bytes >> 4); i += kThreads) dst[i] = src[i];
  }
  if (!in_cache) return;                            // uniform per workgroup

  // first path entry that is not already in place; everything before it stays
  int first = m;
  for (int j = 0; j < m; ++j)
    if (path[j] != j + 1) { first = j; break; }
  if (first == m) return;

  auto row_ptr = [&](void* pool, int pos) -> char* {
    size_t row;
    if (a.paged) {
      const int pg = a.page_table[static_cast<size_t>(b) * a.max_pages + pos / a.page_size];
      if (!page_in_pool(pg, a.n_pages, a.status)) return nullptr;   // a row of a page outside the pool is neither read nor written
      row = (static_cast<size_t>(pg) * a.Hkv + h) * a.page_size + pos % a.page_size;
    } else {
      row = (static_cast<size_t>(b) * a.Hkv + h) * a.l_max + pos;
    }
    return static_cast<char*>(pool) + static_cast<size_t>(layer) * a.layer_stride_bytes + row * a.row_bytes;
  };

  const int rows = m - first;
  const int items = 2 * rows * lpr;                 // K rows then V rows
  uint4 buf[kMaxItems];
#pragma unroll
  for (int u = 0; u < kMaxItems; ++u) {
    const int it = threadIdx.x + u * kThreads;
    if (it < items) {
      const int which = it / (rows * lpr), rem = it % (rows * lpr);
      const int j = first + rem / lpr, piece = rem % lpr;
      const int node = path[j];
      buf[u] = make_uint4(0, 0, 0, 0);
      if (node >= 1 && node < a.n_q) {
        const char* src = row_ptr(which ? a.v : a.k, L + node);
        if (src) buf[u] = reinterpret_cast<const uint4*>(src)[piece];
      } else {
        report_status(a.status, kStatusBadNode);
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int u = 0; u < kMaxItems; ++u) {
    const int it = threadIdx.x + u * kThreads;
    if (it < items) {
      const int which = it / (rows * lpr), rem = it % (rows * lpr);
      const int j = first + rem / lpr, piece = rem % lpr;
      const int node = path[j];
      if (node >= 1 && node < a.n_q) {
        char* dst = row_ptr(which ? a.v : a.k, L + 1 + j);
        if (dst) reinterpret_cast<uint4*>(dst)[piece] = buf[u];
      }
    }
  }
}

}  // namespace

bool kv_compact_supported(const CompactArgs& a) {
  // every piece of every row must fit the per-thread buffer
  return a.row_bytes % 16 == 0 && 2 * (a.n_q - 1) * (a.row_bytes / 16) <= kThreads * kMaxItems;
}

hipError_t launch_kv_compact(const CompactArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(k_kv_compact, dim3(a.Hkv, a.B, a.n_layers), dim3(kThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace sx
