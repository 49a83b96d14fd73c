// Measurement aid: a plain copy of known size that reads through the same load path as the
// weight and KV streams (non-temporal 16-byte loads) or through ordinary loads.  Hardware
// byte counters are scaled by what they report for this kernel.
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

template <bool NT>
__global__ __launch_bounds__(256) void k_copy_probe(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec) {
  size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x;
  const size_t stride = static_cast<size_t>(gridDim.x) * 256;
  for (; i < nvec; i += stride) {
    uint4 v;
    if (NT) {
      const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src + i));
      v = make_uint4(t.x, t.y, t.z, t.w);
    } else {
      v = src[i];
    }
    dst[i] = v;
  }
}

}  // namespace

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, bool nontemporal, hipStream_t s) {
  const size_t nvec = bytes / 16;
  const dim3 grid(8192), block(256);
  if (nontemporal)
    hipLaunchKernelGGL(k_copy_probe<true>, grid, block, 0, s, static_cast<const uint4*>(src), static_cast<uint4*>(dst), nvec);
  else
    hipLaunchKernelGGL(k_copy_probe<false>, grid, block, 0, s, static_cast<const uint4*>(src), static_cast<uint4*>(dst), nvec);
  return hipGetLastError();
}

}  // namespace sx
