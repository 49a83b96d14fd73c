// Verification attention (Alg. 1, "forward through M_t with tree attention"): the draft
// block's n_q queries of every head attend to the whole cached context plus the block
// entries their ancestor mask allows.  The KV cache is read once: all G * n_q query rows
// that share a KV head are processed together, the cache length is cut into chunks that
// run as independent workgroups (each keeps an online softmax), and a second kernel
// merges the chunks' (max, sum, output) triples exactly.
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

constexpr int kTK = 32;  // keys per tile of the ALU kernel

template <typename T>
__device__ __forceinline__ const T* kv_row(const AttnArgs& a, const void* pool, int b, int g, int64_t p) {
  const T* base = static_cast<const T*>(pool);
  if (a.paged) {
    const int page = a.page_table[static_cast<size_t>(b) * a.max_pages + p / a.page_size];
    return base + ((static_cast<size_t>(page) * a.Hkv + g) * a.page_size + p % a.page_size) * a.d;
  }
  return base + ((static_cast<size_t>(b) * a.Hkv + g) * a.l_max + p) * a.d;
}

// Plain-ALU kernel, any storage type: the reference path for fp32 caches.
template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_split_valu(const AttnArgs a) {
  extern __shared__ float smem[];
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int G = a.Hq / a.Hkv;
  const int R = G * a.n_q;
  const int L = a.ctx_len[b];
  const int total = L + a.n_blk;
  const int s0 = split * a.chunk;
  if (s0 >= total) return;
  const int s1 = min(total, s0 + a.chunk);
  constexpr int DP = D + 4;
  float* Qs = smem;                 // [R][D]
  float* Ks = Qs + R * D;           // [kTK][DP]
  float* Vs = Ks + kTK * DP;        // [kTK][DP]
  float* Ss = Vs + kTK * DP;        // [R][kTK]
  float* Ms = Ss + R * kTK;         // [R] running max
  float* Ls = Ms + R;               // [R] running sum
  float* As = Ls + R;               // [R] rescale of this tile
  const int tid = threadIdx.x;

  for (int idx = tid; idx < R * D; idx += 256) {
    const int r = idx / D, c = idx % D;
    const int i = r / G, hh = r % G;
    const T* qp = static_cast<const T*>(a.q) + ((static_cast<size_t>(b) * a.n_q + i) * a.Hq + g * G + hh) * D;
    Qs[idx] = Elem<T>::load(qp + c);
  }
  for (int r = tid; r < R; r += 256) { Ms[r] = -INFINITY; Ls[r] = 0.f; }

  constexpr int C4 = D / 4;               // float4 columns
  constexpr int RSTEP = 256 / C4;         // rows covered per pass
  constexpr int MAXU = (128 + RSTEP - 1) / RSTEP;
  const int c4 = tid % C4, r0 = tid / C4;
  float4 o[MAXU];
#pragma unroll
  for (int u = 0; u < MAXU; ++u) o[u] = make_float4(0.f, 0.f, 0.f, 0.f);
  __syncthreads();

  for (int t0 = s0; t0 < s1; t0 += kTK) {
    // stage K and V rows of this tile as fp32
    for (int idx = tid; idx < kTK * (D / Elem<T>::kPer16B); idx += 256) {
      constexpr int VPR = D / Elem<T>::kPer16B;
      const int j = idx / VPR, vc = idx % VPR;
      const int p = t0 + j;
      float kf[8], vf[8];
      if (p < s1) {
        const uint4 kraw = reinterpret_cast<const uint4*>(kv_row<T>(a, a.k, b, g, p))[vc];
        const uint4 vraw = reinterpret_cast<const uint4*>(kv_row<T>(a, a.v, b, g, p))[vc];
        if (Elem<T>::kPer16B == 8) {
          unpack16(kraw, kf);
          unpack16(vraw, vf);
        } else {
          kf[0] = __uint_as_float(kraw.x); kf[1] = __uint_as_float(kraw.y);
          kf[2] = __uint_as_float(kraw.z); kf[3] = __uint_as_float(kraw.w);
          vf[0] = __uint_as_float(vraw.x); vf[1] = __uint_as_float(vraw.y);
          vf[2] = __uint_as_float(vraw.z); vf[3] = __uint_as_float(vraw.w);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 8; ++e) { kf[e] = 0.f; vf[e] = 0.f; }
      }
#pragma unroll
      for (int e = 0; e < Elem<T>::kPer16B; ++e) {
        Ks[j * DP + vc * Elem<T>::kPer16B + e] = kf[e];
        Vs[j * DP + vc * Elem<T>::kPer16B + e] = vf[e];
      }
    }
    __syncthreads();
    // scores with the block mask applied
    for (int idx = tid; idx < R * kTK; idx += 256) {
      const int r = idx / kTK, j = idx % kTK;
      const int p = t0 + j;
      bool vis = p < s1;
      if (vis && p >= L) {
        const int i = r / G;
        const uint64_t row = a.mask ? a.mask[static_cast<size_t>(b) * a.mask_stride + i] : ((2ull << i) - 1ull);
        vis = (row >> (p - L)) & 1ull;
      }
      float acc = 0.f;
      if (vis) {
        const float4* qv = reinterpret_cast<const float4*>(Qs + r * D);
        const float4* kv = reinterpret_cast<const float4*>(Ks + j * DP);
#pragma unroll 8
        for (int c = 0; c < C4; ++c) {
          const float4 x = qv[c], y = kv[c];
          acc = fmaf(x.x, y.x, acc); acc = fmaf(x.y, y.y, acc);
          acc = fmaf(x.z, y.z, acc); acc = fmaf(x.w, y.w, acc);
        }
      }
      Ss[idx] = vis ? acc * a.scale : -INFINITY;
    }
    __syncthreads();
    // online softmax bookkeeping, one thread per row
    for (int r = tid; r < R; r += 256) {
      float tmax = -INFINITY;
      for (int j = 0; j < kTK; ++j) tmax = fmaxf(tmax, Ss[r * kTK + j]);
      const float m_old = Ms[r];
      const float m_new = fmaxf(m_old, tmax);
      float alpha = 1.f, sum = 0.f;
      if (m_new == -INFINITY) {
        for (int j = 0; j < kTK; ++j) Ss[r * kTK + j] = 0.f;
      } else {
        alpha = (m_old == -INFINITY) ? 0.f : expf(m_old - m_new);
        for (int j = 0; j < kTK; ++j) {
          const float pj = expf(Ss[r * kTK + j] - m_new);  // exp(-inf) = 0 for masked keys
          Ss[r * kTK + j] = pj;
          sum += pj;
        }
      }
      Ms[r] = m_new;
      Ls[r] = Ls[r] * alpha + sum;
      As[r] = alpha;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < MAXU; ++u) {
      const int r = r0 + u * RSTEP;
      if (r < R) {
        const float al = As[r];
        float4 acc = make_float4(o[u].x * al, o[u].y * al, o[u].z * al, o[u].w * al);
        for (int j = 0; j < kTK; ++j) {
          const float pj = Ss[r * kTK + j];
          const float4 vv = *reinterpret_cast<const float4*>(Vs + j * DP + c4 * 4);
          acc.x = fmaf(pj, vv.x, acc.x); acc.y = fmaf(pj, vv.y, acc.y);
          acc.z = fmaf(pj, vv.z, acc.z); acc.w = fmaf(pj, vv.w, acc.w);
        }
        o[u] = acc;
      }
    }
    __syncthreads();
  }
  const size_t unit = (static_cast<size_t>(b) * a.Hkv + g) * a.nsplit + split;
#pragma unroll
  for (int u = 0; u < MAXU; ++u) {
    const int r = r0 + u * RSTEP;
    if (r < R) *reinterpret_cast<float4*>(a.part_o + (unit * R + r) * D + c4 * 4) = o[u];
  }
  for (int r = tid; r < R; r += 256) {
    a.part_ml[(unit * R + r) * 2 + 0] = Ms[r];
    a.part_ml[(unit * R + r) * 2 + 1] = Ls[r];
  }
}

// Merge the chunks of one (sequence, query, head): exact log-sum-exp combination.  One
// workgroup per output row: the chunks' weights exp(m_s - max) are formed once in LDS, then
// the threads split into groups that each take every NG-th chunk of one float4 column, so
// all partial outputs are requested at once; the groups are added in a fixed order.
constexpr int kCombThreads = 256;

template <typename T, int D>
__global__ __launch_bounds__(kCombThreads) void k_attn_combine(const AttnArgs a) {
  constexpr int C4 = D / 4;                 // float4 columns of a row
  constexpr int NG = kCombThreads / C4;     // chunk groups
  extern __shared__ float w_lds[];          // [nsplit] weights, then NG x C4 float4 for the group sums
  __shared__ float red[kCombThreads / 64];
  const int h = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
  const int G = a.Hq / a.Hkv;
  const int R = G * a.n_q;
  const int g = h / G, r = i * G + h % G;
  const int total = a.ctx_len[b] + a.n_blk;
  const int nact = min((total + a.chunk - 1) / a.chunk, a.nsplit);
  const size_t unit0 = (static_cast<size_t>(b) * a.Hkv + g) * a.nsplit;
  const float* ml = a.part_ml + (unit0 * R + r) * 2;          // chunk s at ml[s * R * 2]
  const float* po = a.part_o + (unit0 * R + r) * D;            // chunk s at po[s * R * D]
  float mloc = -INFINITY;
  for (int s = threadIdx.x; s < nact; s += kCombThreads) mloc = fmaxf(mloc, ml[static_cast<size_t>(s) * R * 2]);
  mloc = wave_max(mloc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mloc;
  __syncthreads();
  float mmax = red[0];
#pragma unroll
  for (int w = 1; w < kCombThreads / 64; ++w) mmax = fmaxf(mmax, red[w]);
  __syncthreads();
  float dloc = 0.f;
  for (int s = threadIdx.x; s < nact; s += kCombThreads) {
    const float ms = ml[static_cast<size_t>(s) * R * 2];
    float w = 0.f;
    if (ms != -INFINITY) w = a.use_mfma ? exp2f(ms - mmax) : expf(ms - mmax);
    w_lds[s] = w;
    dloc = fmaf(w, w != 0.f ? ml[static_cast<size_t>(s) * R * 2 + 1] : 0.f, dloc);
  }
  dloc = wave_sum(dloc);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = dloc;
  __syncthreads();
  float den = 0.f;
#pragma unroll
  for (int w = 0; w < kCombThreads / 64; ++w) den += red[w];
  const int sg = threadIdx.x / C4, c4 = threadIdx.x % C4;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = sg; s < nact; s += 4 * NG) {
    float4 o[4];
    float w[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int ss = min(s + u * NG, nact - 1);
      w[u] = s + u * NG < nact ? w_lds[ss] : 0.f;
      o[u] = *reinterpret_cast<const float4*>(po + static_cast<size_t>(ss) * R * D + c4 * 4);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (w[u] != 0.f) {
        acc.x = fmaf(w[u], o[u].x, acc.x); acc.y = fmaf(w[u], o[u].y, acc.y);
        acc.z = fmaf(w[u], o[u].z, acc.z); acc.w = fmaf(w[u], o[u].w, acc.w);
      }
  }
  float4* gs = reinterpret_cast<float4*>(w_lds + ((a.nsplit + 3) & ~3));
  gs[sg * C4 + c4] = acc;
  __syncthreads();
  if (sg == 0) {
    float4 sum = gs[c4];
    for (int u = 1; u < NG; ++u) {
      const float4 v = gs[u * C4 + c4];
      sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
    }
    T* dst = static_cast<T*>(a.out) + ((static_cast<size_t>(b) * a.n_q + i) * a.Hq + h) * D + c4 * 4;
    Elem<T>::store(dst + 0, sum.x / den); Elem<T>::store(dst + 1, sum.y / den);
    Elem<T>::store(dst + 2, sum.z / den); Elem<T>::store(dst + 3, sum.w / den);
  }
}

size_t valu_smem_bytes(const AttnArgs& a) {
  const int R = (a.Hq / a.Hkv) * a.n_q;
  return sizeof(float) * (static_cast<size_t>(R) * a.d + 2 * kTK * (a.d + 4) + static_cast<size_t>(R) * kTK + 3 * R);
}

template <typename T, int D>
hipError_t launch_valu(const AttnArgs& a, hipStream_t s) {
  const size_t smem = valu_smem_bytes(a);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_split_valu<T, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((k_attn_split_valu<T, D>), dim3(a.nsplit, a.Hkv, a.B), dim3(256), smem, s, a);
  return hipGetLastError();
}

}  // namespace

void attn_plan(AttnArgs& a, int num_cus) {
  // Chunk of the cache length handled by one workgroup.  The host knows only the upper
  // bound l_max of the lengths, so the grid is sized for it and workgroups past a sequence's
  // end leave at once.  Small problems get one workgroup per CU at most (a second round of
  // workgroups would double their latency); large ones get about three rounds so that
  // sequences of different length balance out.
  a.use_mfma = attn_mfma_supported(a) ? 1 : 0;
  const int64_t units = static_cast<int64_t>(a.B) * a.Hkv;
  const int64_t lmax = a.l_max;
  const int64_t keys = units * lmax;
  const int64_t rounds = keys >= static_cast<int64_t>(num_cus) * 3 * 1024 ? 3 : 1;
  const int64_t per_cu = a.use_mfma ? 2 : 1;   // workgroups of the matrix-core kernel that fit a CU
  const int64_t target = rounds * num_cus * (rounds == 1 ? per_cu : 1);
  int64_t chunk = (keys + target - 1) / target;
  chunk = ((chunk + 127) / 128) * 128;
  if (chunk < 128) chunk = 128;
  // never more workgroups than the target: rounding the split count up must not spill over
  while (units * ((lmax + chunk - 1) / chunk) > target && chunk < lmax) chunk += 128;
  if (a.use_mfma && chunk > attn_mfma_max_chunk(a)) chunk = attn_mfma_max_chunk(a) / 128 * 128;
  a.chunk = static_cast<int>(chunk);
  a.nsplit = static_cast<int>((lmax + chunk - 1) / chunk);
  if (a.nsplit < 1) a.nsplit = 1;
}

size_t attn_workspace_bytes(const AttnArgs& a) {
  const size_t R = static_cast<size_t>(a.Hq / a.Hkv) * a.n_q;
  const size_t units = static_cast<size_t>(a.B) * a.Hkv * a.nsplit;
  size_t o = units * R * a.d * sizeof(float);
  o = (o + 255) & ~static_cast<size_t>(255);
  size_t ml = units * R * 2 * sizeof(float);
  ml = (ml + 255) & ~static_cast<size_t>(255);
  return o + ml;
}

hipError_t launch_attn(const AttnArgs& a, hipStream_t s, KernelHook hook, int hook_id) {
  hipError_t e;
  if (hook) hook(hook_id, 0, s);
  if (a.use_mfma) {
    e = launch_attn_mfma(a, s);
  } else if (a.dtype == 1) {
    e = a.d == 128 ? launch_valu<bf16_t, 128>(a, s) : launch_valu<bf16_t, 64>(a, s);
  } else {
    e = a.d == 128 ? launch_valu<float, 128>(a, s) : launch_valu<float, 64>(a, s);
  }
  if (hook) hook(hook_id, 1, s);
  if (e != hipSuccess) return e;
  const dim3 grid(a.Hq, a.n_q, a.B);
  const size_t lds = (static_cast<size_t>((a.nsplit + 3) & ~3) + kCombThreads * 4) * sizeof(float);
  if (lds > 60 * 1024) return hipErrorInvalidValue;
  if (a.dtype == 1) {
    if (a.d == 128) hipLaunchKernelGGL((k_attn_combine<bf16_t, 128>), grid, dim3(kCombThreads), lds, s, a);
    else hipLaunchKernelGGL((k_attn_combine<bf16_t, 64>), grid, dim3(kCombThreads), lds, s, a);
  } else {
    if (a.d == 128) hipLaunchKernelGGL((k_attn_combine<float, 128>), grid, dim3(kCombThreads), lds, s, a);
    else hipLaunchKernelGGL((k_attn_combine<float, 64>), grid, dim3(kCombThreads), lds, s, a);
  }
  return hipGetLastError();
}

}  // namespace sx
