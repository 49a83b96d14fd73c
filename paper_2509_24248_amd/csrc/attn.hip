// Verification attention (Alg. 1, the target's verification forward over the draft block): the
// block's n_q queries of every head attend to the whole cached context plus the block
// entries their ancestor mask allows.  The KV cache is read once: all G * n_q query rows
// that share a KV head are processed together, the keys of all sequences are dealt to the
// workgroups in equal shares (attn_sched.hpp; each segment keeps an online softmax), and a
// second kernel merges the segments' (max, sum, output) triples exactly.
#include "attn_sched.hpp"
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

constexpr int kTK = 32;  // keys per tile of the ALU kernel

template <typename T>
__device__ __forceinline__ const T* kv_row(const AttnArgs& a, const void* pool, int b, int g, int64_t p) {
  const T* base = static_cast<const T*>(pool);
  if (a.paged) {
    const int page = checked_page(a.page_table[static_cast<size_t>(b) * a.max_pages + p / a.page_size], a.n_pages, a.status);
    return base + ((static_cast<size_t>(page) * a.Hkv + g) * a.page_size + p % a.page_size) * a.d;
  }
  return base + ((static_cast<size_t>(b) * a.Hkv + g) * a.l_max + p) * a.d;
}

// Plain-ALU kernel, any storage type: the reference path for fp32 caches.
template <typename T, int D>
__global__ __launch_bounds__(256) void k_attn_split_valu(const AttnArgs a) {
  extern __shared__ float smem[];
  const int G = a.Hq / a.Hkv;
  const int R = G * a.n_q;
  const int tid = threadIdx.x;
  constexpr int DP = D + 4;
  float* Qs = smem;                 // [R][D]
  float* Ks = Qs + R * D;           // [kTK][DP]
  float* Vs = Ks + kTK * DP;        // [kTK][DP]
  float* Ss = Vs + kTK * DP;        // [R][kTK]
  float* Ms = Ss + R * kTK;         // [R] running max
  float* Ls = Ms + R;               // [R] running sum
  float* As = Ls + R;               // [R] rescale of this tile
  int* sched_lds = reinterpret_cast<int*>(As + R);   // [B + 1]
  attn_sched_build(a, sched_lds);
  const int Tg = a.Hkv * sched_lds[a.B];     // granules on the line
  const int W = attn_sched_workgroups(Tg, a.wgrid);
  if (blockIdx.x == 0) {
    for (int i = tid; i <= a.B; i += 256) a.sched[i] = sched_lds[i];
    if (tid == 0) a.sched[a.B + 1] = W;
  }
  if (static_cast<int>(blockIdx.x) >= W) return;
  const int x_hi = attn_sched_lo(blockIdx.x + 1, Tg, W);
  for (int x_cur = attn_sched_lo(blockIdx.x, Tg, W); x_cur < x_hi;) {
  const AttnSeg seg = attn_sched_segment(a, sched_lds, x_cur, x_hi);
  x_cur = seg.next;
  const int g = seg.g, b = seg.b, L = seg.L, s0 = seg.s0, s1 = seg.s1;

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
  const size_t unit = static_cast<size_t>(blockIdx.x) + static_cast<size_t>(b) * a.Hkv + g;   // partial slot of segment (w, u)
#pragma unroll
  for (int u = 0; u < MAXU; ++u) {
    const int r = r0 + u * RSTEP;
    if (r < R) *reinterpret_cast<float4*>(a.part_o + (unit * R + r) * D + c4 * 4) = o[u];
  }
  for (int r = tid; r < R; r += 256) {
    a.part_ml[(unit * R + r) * 2 + 0] = Ms[r];
    a.part_ml[(unit * R + r) * 2 + 1] = Ls[r];
  }
  __syncthreads();   // a further segment restarts the running maxima and sums
  }
}

// Merge the segments of one (sequence, query, head): exact log-sum-exp combination.  One
// workgroup per output row: the chunks' weights exp(m_s - max) are formed once in LDS, then
// the threads split into groups that each take every NG-th chunk of one float4 column, so
// all partial outputs are requested at once; the groups are added in a fixed order.
constexpr int kCombThreads = 256;

template <typename T, int D>
__global__ __launch_bounds__(kCombThreads) void k_attn_combine(const AttnArgs a) {
  constexpr int C4 = D / 4;                 // float4 columns of a row
  constexpr int NG = kCombThreads / C4;     // chunk groups
  extern __shared__ float w_lds[];          // [wgrid] weights (a unit has at most that many segments), then NG x C4 float4 for the group sums
  __shared__ float red[kCombThreads / 64];
  const int h = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
  const int G = a.Hq / a.Hkv;
  const int R = G * a.n_q;
  const int g = h / G, r = i * G + h % G;
  // the segments of this row's unit: consecutive slots, one per workgroup whose range touched it
  const int n_b = a.sched[b + 1] - a.sched[b];
  const int Tg = a.Hkv * a.sched[a.B], W = a.sched[a.B + 1];
  const int p_u = a.Hkv * a.sched[b] + g * n_b;
  const int w_first = attn_sched_owner(p_u, Tg, W);
  const int nact = attn_sched_owner(p_u + n_b - 1, Tg, W) - w_first + 1;
  const size_t unit0 = static_cast<size_t>(w_first) + static_cast<size_t>(b) * a.Hkv + g;
  const float* ml = a.part_ml + (unit0 * R + r) * 2;          // segment s at ml[s * R * 2]
  const float* po = a.part_o + (unit0 * R + r) * D;            // segment s at po[s * R * D]
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
  float4* gs = reinterpret_cast<float4*>(w_lds + ((a.wgrid + 3) & ~3));
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
  return sizeof(float) * (static_cast<size_t>(R) * a.d + 2 * kTK * (a.d + 4) + static_cast<size_t>(R) * kTK + 3 * R + a.B + 1);
}

template <typename T, int D>
hipError_t launch_valu(const AttnArgs& a, hipStream_t s) {
  const size_t smem = valu_smem_bytes(a);
  // set once per process; a function-local static is initialised under the language's own lock,
  // so first calls from several host threads are safe
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_split_valu<T, D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((k_attn_split_valu<T, D>), dim3(a.wgrid), dim3(256), smem, s, a);
  return hipGetLastError();
}

}  // namespace

constexpr size_t kCombineLdsMax = 60 * 1024;

size_t combine_lds_bytes(int wgrid) { return (static_cast<size_t>((wgrid + 3) & ~3) + kCombThreads * 4) * sizeof(float); }

bool attn_plan(AttnArgs& a, int num_cus) {
  // The host knows only the upper bound l_max of the lengths; the kernels deal the keys that
  // are really there to the workgroups in equal shares.  Here only the number of workgroups is
  // set: as many as are resident at once (one or two of the matrix-core kernel per compute unit),
  // fewer when even the longest possible caches would leave them less than two granules (128
  // keys) each, more when a share could otherwise exceed what one segment can hold.
  a.use_mfma = attn_mfma_supported(a) ? 1 : 0;
  if (a.B > kAttnMaxSeqs || a.l_max < a.n_blk) return false;
  const int64_t units = static_cast<int64_t>(a.B) * a.Hkv;
  const int64_t gmax = (a.l_max + kAttnGran - 1) / kAttnGran;      // granules of the longest possible unit
  const int64_t tmax = units * gmax;
  if (tmax >= (1ll << 30)) return false;
  a.stages = a.use_mfma ? attn_mfma_stages(a) : 0;
  const int64_t resident = static_cast<int64_t>(num_cus) * (a.use_mfma ? attn_mfma_per_cu(a) : 1);
  int64_t w = tmax / 2 < resident ? tmax / 2 : resident;
  if (w < 1) w = 1;
  if (a.use_mfma) {
    const int64_t seg_gran = attn_mfma_max_chunk(a) / kAttnGran;   // granules one segment may span
    const int64_t need = (tmax + seg_gran - 1) / seg_gran;
    if (w < need) w = need;
  }
  if (combine_lds_bytes(static_cast<int>(w)) > kCombineLdsMax) return false;
  a.wgrid = static_cast<int>(w);
  return true;
}

int attn_slots(const AttnArgs& a) { return a.wgrid + a.B * a.Hkv; }

size_t attn_workspace_bytes(const AttnArgs& a) {
  const size_t R = static_cast<size_t>(a.Hq / a.Hkv) * a.n_q;
  const size_t slots = static_cast<size_t>(attn_slots(a));
  size_t o = slots * R * a.d * sizeof(float);
  o = (o + 255) & ~static_cast<size_t>(255);
  size_t ml = slots * R * 2 * sizeof(float);
  ml = (ml + 255) & ~static_cast<size_t>(255);
  size_t sc = static_cast<size_t>(a.B + 2) * sizeof(int);
  sc = (sc + 255) & ~static_cast<size_t>(255);
  return o + ml + sc;
}

void attn_carve(AttnArgs& a, void* workspace) {
  const size_t R = static_cast<size_t>(a.Hq / a.Hkv) * a.n_q;
  const size_t slots = static_cast<size_t>(attn_slots(a));
  char* p = static_cast<char*>(workspace);
  a.part_o = reinterpret_cast<float*>(p);
  p += (slots * R * a.d * sizeof(float) + 255) & ~static_cast<size_t>(255);
  a.part_ml = reinterpret_cast<float*>(p);
  p += (slots * R * 2 * sizeof(float) + 255) & ~static_cast<size_t>(255);
  a.sched = reinterpret_cast<int*>(p);
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
  const size_t lds = combine_lds_bytes(a.wgrid);   // attn_plan made sure it fits
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
