// Row-wise glue of the draft step (Sec. 3.1; Alg. 1 first loop line): everything between
// the weight-streaming GEMMs.  Each kernel reduces the split-K partial sums of the GEMM
// before it, applies the layer's elementwise math in fp32 and emits the next GEMM's
// activations as fp32 rows (the MFMA GEMM splits them into bf16 hi + lo parts itself).
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

// sum over split-K ranges and planes of 8 consecutive outputs of row b
__device__ __forceinline__ void gather_partial(const float* partial, int nslices, int planes, int B,
                                               int N, int b, int n, float (&f)[8]) {
  const int Mv = B * planes;
#pragma unroll
  for (int e = 0; e < 8; ++e) f[e] = 0.f;
  for (int ks = 0; ks < nslices; ++ks) {
    for (int p = 0; p < planes; ++p) {
      const float4* src = reinterpret_cast<const float4*>(
          partial + (static_cast<size_t>(ks) * Mv + b * planes + p) * N + n);
      const float4 a = src[0], c = src[1];
      f[0] += a.x; f[1] += a.y; f[2] += a.z; f[3] += a.w;
      f[4] += c.x; f[5] += c.y; f[6] += c.z; f[7] += c.w;
    }
  }
}

template <typename T>
__global__ __launch_bounds__(256) void k_embed_concat(int D, int V, int* status, const T* __restrict__ embed,
                                                      const int32_t* __restrict__ tok,
                                                      const T* __restrict__ hidden_in,
                                                      float* __restrict__ act) {
  const int b = blockIdx.x;
  const T* e = embed + static_cast<size_t>(checked_token(tok[b], V, status)) * D;
  const T* h = hidden_in + static_cast<size_t>(b) * D;
  for (int g8 = threadIdx.x; g8 < 2 * D / 8; g8 += 256) {
    const int k = g8 * 8;
    const T* src = k < D ? e + k : h + (k - D);
    float f[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) f[i] = Elem<T>::load(src + i);
#pragma unroll
    for (int i = 0; i < 8; ++i) act[static_cast<size_t>(b) * 2 * D + k + i] = f[i];
  }
}

constexpr int kNormThreads = 1024;
constexpr int kNormIters = 2;   // float4 per thread per iteration: rows up to 2 * 1024 * 4 = 8192 wide

template <typename T>
__global__ __launch_bounds__(kNormThreads) void k_reduce_norm(int B, int N, const float* __restrict__ partial,
                                                              int nslices, int planes,
                                                              const float* __restrict__ residual,
                                                              const T* __restrict__ gain, float eps,
                                                              float* __restrict__ sum_out, T* __restrict__ hidden_out,
                                                              float* __restrict__ act) {
  __shared__ float sh[kNormThreads / 64];
  const int b = blockIdx.x;
  const int Mv = B * planes;
  const int total = nslices * planes;   // partial rows to add: slice j -> row (j / planes) * Mv + b * planes + j % planes
  float4 vals[kNormIters];
  float ssq = 0.f;
#pragma unroll
  for (int it = 0; it < kNormIters; ++it) {
    const int n = (threadIdx.x + it * kNormThreads) * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n < N) {
      if (residual) acc = *reinterpret_cast<const float4*>(residual + static_cast<size_t>(b) * N + n);
      int j = 0;
      for (; j + 4 <= total; j += 4) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int jj = j + u;
          const size_t row = static_cast<size_t>(jj / planes) * Mv + b * planes + jj % planes;
          v[u] = *reinterpret_cast<const float4*>(partial + row * N + n);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
      }
      for (; j < total; ++j) {
        const size_t row = static_cast<size_t>(j / planes) * Mv + b * planes + j % planes;
        const float4 v = *reinterpret_cast<const float4*>(partial + row * N + n);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
      ssq += acc.x * acc.x + acc.y * acc.y + acc.z * acc.z + acc.w * acc.w;
      if (sum_out) *reinterpret_cast<float4*>(sum_out + static_cast<size_t>(b) * N + n) = acc;
      if (hidden_out) {
        T* dst = hidden_out + static_cast<size_t>(b) * N + n;
        Elem<T>::store(dst + 0, acc.x); Elem<T>::store(dst + 1, acc.y);
        Elem<T>::store(dst + 2, acc.z); Elem<T>::store(dst + 3, acc.w);
      }
    }
    vals[it] = acc;
  }
  ssq = wave_sum(ssq);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = ssq;
  __syncthreads();
  float tot = 0.f;
#pragma unroll
  for (int w = 0; w < kNormThreads / 64; ++w) tot += sh[w];
  const float rinv = 1.0f / sqrtf(tot / static_cast<float>(N) + eps);
#pragma unroll
  for (int it = 0; it < kNormIters; ++it) {
    const int n = (threadIdx.x + it * kNormThreads) * 4;
    if (n < N) {
      float4 o;
      o.x = vals[it].x * rinv * Elem<T>::load(gain + n + 0);
      o.y = vals[it].y * rinv * Elem<T>::load(gain + n + 1);
      o.z = vals[it].z * rinv * Elem<T>::load(gain + n + 2);
      o.w = vals[it].w * rinv * Elem<T>::load(gain + n + 3);
      *reinterpret_cast<float4*>(act + static_cast<size_t>(b) * N + n) = o;
    }
  }
}

// Row r of the step belongs to sequence r / W.  Its rotary position is pos[r / W] + level and
// its K/V go to cache entry pos[r / W] + node[r % W] (chain step: W = 1, level 0, node null
// = entry pos itself; tree level: position = context + depth, entry = context + node id).
template <typename T>
__global__ void k_rope_kvwrite(int M, int W, int Hq, int Hkv, int d, const float* __restrict__ partial,
                               int nslices, int planes, const int32_t* __restrict__ pos, int level,
                               const int32_t* __restrict__ node, float theta,
                               T* __restrict__ q_out, int paged, T* __restrict__ kc, T* __restrict__ vc,
                               const int32_t* __restrict__ page_table, int page_size, int max_pages,
                               int64_t l_max, int64_t n_pages, int* status) {
  const int r = blockIdx.x, hh = blockIdx.y, c = threadIdx.x;  // c in [0, d/2)
  const int b = r / W;
  const int N = (Hq + 2 * Hkv) * d;
  const int Mv = M * planes;
  const int half = d >> 1;
  float x1 = 0.f, x2 = 0.f;
  for (int ks = 0; ks < nslices; ++ks)
    for (int p = 0; p < planes; ++p) {
      const float* src = partial + (static_cast<size_t>(ks) * Mv + r * planes + p) * N + hh * d;
      x1 += src[c];
      x2 += src[c + half];
    }
  const int ps = pos[b] + level;
  const int slot = pos[b] + (node ? node[r % W] : 0);
  if (hh < Hq + Hkv) {
    // rotary embedding, pairing (c, c + d/2); the angle is formed in double so that long
    // positions keep their phase
    const double inv = pow(static_cast<double>(theta), -2.0 * c / d);
    const double ang = static_cast<double>(ps) * inv;
    const float cs = static_cast<float>(cos(ang)), sn = static_cast<float>(sin(ang));
    const float r1 = x1 * cs - x2 * sn;
    const float r2 = x2 * cs + x1 * sn;
    x1 = r1;
    x2 = r2;
  }
  if (hh < Hq) {
    T* dst = q_out + (static_cast<size_t>(r) * Hq + hh) * d;
    Elem<T>::store(dst + c, x1);
    Elem<T>::store(dst + c + half, x2);
    return;
  }
  if (slot < 0 || slot >= l_max) return;       // an entry outside the cache is not written
  const bool is_k = hh < Hq + Hkv;
  const int h = is_k ? hh - Hq : hh - Hq - Hkv;
  size_t off;
  if (paged) {
    const int page = page_table[static_cast<size_t>(b) * max_pages + slot / page_size];
    if (!page_in_pool(page, n_pages, status)) return;
    off = ((static_cast<size_t>(page) * Hkv + h) * page_size + slot % page_size) * d;
  } else {
    off = ((static_cast<size_t>(b) * Hkv + h) * l_max + slot) * d;
  }
  T* dst = (is_k ? kc : vc) + off;
  Elem<T>::store(dst + c, x1);
  Elem<T>::store(dst + c + half, x2);
}

__global__ __launch_bounds__(256) void k_silu_mul(int B, int I, const float* __restrict__ partial,
                                                  int nslices, int planes, float* __restrict__ act) {
  const int b = blockIdx.x;
  for (int g8 = blockIdx.y * 256 + threadIdx.x; g8 < I / 8; g8 += 256 * gridDim.y) {
    float gt[8], up[8], f[8];
    gather_partial(partial, nslices, planes, B, 2 * I, b, g8 * 8, gt);
    gather_partial(partial, nslices, planes, B, 2 * I, b, I + g8 * 8, up);
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = gt[e] * sigmoidf_(gt[e]) * up[e];
#pragma unroll
    for (int e = 0; e < 8; ++e) act[static_cast<size_t>(b) * I + g8 * 8 + e] = f[e];
  }
}

__global__ void k_head_finalize(int B, int rem_activation, const int32_t* __restrict__ argmax_in,
                                const float* __restrict__ extra, int32_t* __restrict__ next_tok,
                                float* __restrict__ sig_raw, float* __restrict__ sig) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  next_tok[b] = argmax_in[b];
  const float zc = extra[b * 3 + 0], zp = extra[b * 3 + 1], zr = extra[b * 3 + 2];
  sig_raw[b * 3 + 0] = zc;
  sig_raw[b * 3 + 1] = zp;
  sig_raw[b * 3 + 2] = zr;
  // confidence and progress pass through a sigmoid (Eqs. 3-4); the remaining-length head
  // regresses log(1 + r) (Eq. 5), so r = expm1(z), floored at zero
  sig[b * 3 + 0] = sigmoidf_(zc);
  sig[b * 3 + 1] = sigmoidf_(zp);
  float r;
  if (rem_activation == 0)
    r = fmaxf(0.f, expm1f(zr));
  else if (rem_activation == 1)
    r = sigmoidf_(zr);
  else
    r = zr;
  sig[b * 3 + 2] = r;
}

}  // namespace

hipError_t launch_embed_concat(const DraftDims& dm, int B, const void* embed, const int32_t* tok,
                               const void* hidden_in, float* act, hipStream_t s, int* status) {
  if (dm.dtype == 1)
    hipLaunchKernelGGL(k_embed_concat<bf16_t>, dim3(B), dim3(256), 0, s, dm.D, dm.V, status, static_cast<const bf16_t*>(embed),
                       tok, static_cast<const bf16_t*>(hidden_in), act);
  else
    hipLaunchKernelGGL(k_embed_concat<float>, dim3(B), dim3(256), 0, s, dm.D, dm.V, status, static_cast<const float*>(embed),
                       tok, static_cast<const float*>(hidden_in), act);
  return hipGetLastError();
}

hipError_t launch_reduce_norm(const DraftDims& dm, int B, int N, const float* partial, int nslices,
                              int planes, const float* residual, const void* gain, float* sum_out,
                              void* hidden_out, float* act, hipStream_t s) {
  if (dm.dtype == 1)
    hipLaunchKernelGGL(k_reduce_norm<bf16_t>, dim3(B), dim3(kNormThreads), 0, s, B, N, partial, nslices, planes, residual,
                       static_cast<const bf16_t*>(gain), dm.rms_eps, sum_out, static_cast<bf16_t*>(hidden_out), act);
  else
    hipLaunchKernelGGL(k_reduce_norm<float>, dim3(B), dim3(kNormThreads), 0, s, B, N, partial, nslices, planes, residual,
                       static_cast<const float*>(gain), dm.rms_eps, sum_out, static_cast<float*>(hidden_out), act);
  return hipGetLastError();
}

hipError_t launch_rope_kvwrite(const DraftDims& dm, int M, int W, const float* partial, int nslices,
                               int planes, const int32_t* pos, int level, const int32_t* node, void* q_out,
                               int kv_paged, void* kc, void* vc, const int32_t* page_table, int page_size,
                               int max_pages, int64_t l_max, hipStream_t s, int64_t n_pages, int* status) {
  const dim3 grid(M, dm.Hq + 2 * dm.Hkv), block(dm.d / 2);
  if (dm.dtype == 1)
    hipLaunchKernelGGL(k_rope_kvwrite<bf16_t>, grid, block, 0, s, M, W, dm.Hq, dm.Hkv, dm.d, partial, nslices, planes,
                       pos, level, node, dm.rope_theta, static_cast<bf16_t*>(q_out), kv_paged,
                       static_cast<bf16_t*>(kc), static_cast<bf16_t*>(vc), page_table, page_size, max_pages, l_max, n_pages, status);
  else
    hipLaunchKernelGGL(k_rope_kvwrite<float>, grid, block, 0, s, M, W, dm.Hq, dm.Hkv, dm.d, partial, nslices, planes,
                       pos, level, node, dm.rope_theta, static_cast<float*>(q_out), kv_paged,
                       static_cast<float*>(kc), static_cast<float*>(vc), page_table, page_size, max_pages, l_max, n_pages, status);
  return hipGetLastError();
}

hipError_t launch_silu_mul(const DraftDims& dm, int B, const float* partial, int nslices, int planes,
                           float* act, hipStream_t s) {
  const int gy = (dm.I / 8 + 255) / 256;
  hipLaunchKernelGGL(k_silu_mul, dim3(B, gy), dim3(256), 0, s, B, dm.I, partial, nslices, planes, act);
  return hipGetLastError();
}

hipError_t launch_head_finalize(const DraftDims& dm, int B, const int32_t* argmax_in, const float* extra,
                                int32_t* next_tok, float* sig_raw, float* sig, hipStream_t s) {
  hipLaunchKernelGGL(k_head_finalize, dim3(1), dim3(64), 0, s, B, dm.rem_activation, argmax_in, extra, next_tok,
                     sig_raw, sig);
  return hipGetLastError();
}

}  // namespace sx
