// Skinny weight-streaming GEMMs  out[m][n] = sum_k act[m][k] * w[n][k]  (M <= 144 rows),
// used for the draft layer's projections, the widened head (Eq. 1) and the target LM head.
// They are HBM-bound: every weight byte is read once, with 16-byte loads coalesced along K.
//
//  k_gemv_valu  : plain fp32 ALU path (fp32 weights, or any shape the MFMA path rejects).
//  k_gemm_mfma  : bf16 path.  One wave owns a 16-row weight tile over a K range.  Weight
//                 rows arrive as 256-byte coalesced segments, pass through a wave-private,
//                 XOR-swizzled LDS tile to reach the MFMA operand layout (row = lane % 16,
//                 8 consecutive k per lane) and are contracted with pre-packed activation
//                 fragments by v_mfma_f32_16x16x32_bf16.  The argmax over the vocabulary is
//                 fused into the epilogue, so logits are never written.
#include "common.hpp"
#include "kernels.hpp"

#include <limits.h>

namespace sx {

namespace {

struct SegRef {
  const char* base;  // first row of the segment
  int row0;          // its first logical row
  int rows;          // rows in the segment
};

__device__ __forceinline__ SegRef find_segment(const GemmArgs& g, int n) {
  SegRef r;
  int start = 0;
  int s = 0;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    if (s + 1 < g.nseg && n >= g.seg_end[s]) {
      start = g.seg_end[s];
      ++s;
    }
  }
  r.base = static_cast<const char*>(g.w[s]);
  r.row0 = start;
  r.rows = g.seg_end[s] - start;
  return r;
}

// ------------------------------------------------------------------------- VALU path
template <typename WT>
__global__ __launch_bounds__(256) void k_gemv_valu(const GemmArgs g) {
  constexpr int EPV = Elem<WT>::kPer16B;
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= g.N) return;
  const SegRef sg = find_segment(g, n);
  const uint4* wrow = reinterpret_cast<const uint4*>(sg.base + static_cast<size_t>(n - sg.row0) * g.K * sizeof(WT));
  const int nvec = g.K / EPV;
  for (int m0 = 0; m0 < g.M; m0 += 8) {
    const int mc = min(8, g.M - m0);
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    for (int c = lane; c < nvec; c += 64) {
      const uint4 wv = wrow[c];
      float wf[8];
      if (EPV == 8) {
        unpack16(wv, wf);
      } else {
        wf[0] = __uint_as_float(wv.x); wf[1] = __uint_as_float(wv.y);
        wf[2] = __uint_as_float(wv.z); wf[3] = __uint_as_float(wv.w);
      }
#pragma unroll
      for (int mm = 0; mm < 8; ++mm) {
        if (mm < mc) {
          const float* a = g.act + static_cast<size_t>(m0 + mm) * g.K + static_cast<size_t>(c) * EPV;
#pragma unroll
          for (int e = 0; e < EPV; e += 4) {
            const float4 av = *reinterpret_cast<const float4*>(a + e);
            acc[mm] = fmaf(av.x, wf[e + 0], acc[mm]);
            acc[mm] = fmaf(av.y, wf[e + 1], acc[mm]);
            acc[mm] = fmaf(av.z, wf[e + 2], acc[mm]);
            acc[mm] = fmaf(av.w, wf[e + 3], acc[mm]);
          }
        }
      }
    }
#pragma unroll
    for (int mm = 0; mm < 8; ++mm) {
      if (mm < mc) {
        const float v = wave_sum(acc[mm]);
        if (lane == 0) g.partial[static_cast<size_t>(m0 + mm) * g.N + n] = v;
      }
    }
  }
}

// ------------------------------------------------------------------------- MFMA path
template <int MT, int PLANES, bool HEAD>
__global__ __launch_bounds__(256) void k_gemm_mfma(const GemmArgs g) {
  // one 16-row x 128-k weight tile (4 KB) per wave; entry [row][pos] holds the 16-byte
  // chunk (pos ^ row) of that row, so both the coalesced writes and the per-row operand
  // reads touch 16 distinct 16-byte slots
  __shared__ uint4 lds[4][256];
  const int lane = threadIdx.x & 63;
  const int wv = threadIdx.x >> 6;
  const int ntiles = (g.N + 15) >> 4;
  const int tile = blockIdx.x * 4 + wv;
  if (tile >= ntiles) return;  // waves are independent: no block-level barrier below
  const int ks = blockIdx.y;
  const int KB = g.K >> 7;
  const int kb0 = ks * g.kb_per_split;
  const int kb1 = min(KB, kb0 + g.kb_per_split);
  const int n0 = tile << 4;
  const SegRef sg = find_segment(g, n0);
  const size_t row_bytes = static_cast<size_t>(g.K) * 2;

  const int pos = lane & 15;
  const char* src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 4 * i + (lane >> 4);
    const int lr = min(n0 - sg.row0 + r, sg.rows - 1);  // clamp: rows past the end are masked later
    src[i] = sg.base + static_cast<size_t>(lr) * row_bytes + static_cast<size_t>((pos ^ r) << 4);
  }
  const int fr = lane & 15, fq = lane >> 4;
  uint4* my = lds[wv];

  f32x4_t acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  const uint4* ap = g.apack + (static_cast<size_t>(kb0) * 4 * MT) * 64 + lane;
  for (int kb = kb0; kb < kb1; ++kb) {
    uint4 wr[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      wr[i] = *reinterpret_cast<const uint4*>(src[i] + (static_cast<size_t>(kb) << 8));
#pragma unroll
    for (int i = 0; i < 4; ++i) my[(4 * i + (lane >> 4)) * 16 + pos] = wr[i];
    // the tile is private to this wave, whose LDS operations retire in order: a compiler
    // fence is all that separates the writes from the transposed reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint4 wf = my[fr * 16 + ((4 * s + fq) ^ fr)];
      const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, wf);
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const uint4 af = ap[(s * MT + t) * 64];
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8_t, af), acc[t], 0, 0, 0);
      }
    }
    ap += 4 * MT * 64;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // accumulator layout: lane (c = lane % 16, q = lane / 16) holds rows n0 + 4q + i of
  // activation column 16 t + c
  const int Mv = g.M * PLANES;
  if (!HEAD) {
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int v = 16 * t + fr;
      if (v < Mv) {
        float* dst = g.partial + (static_cast<size_t>(ks) * Mv + v) * g.N + n0 + 4 * fq;
        if (n0 + 4 * fq + 3 < g.N && (g.N & 3) == 0) {
          *reinterpret_cast<float4*>(dst) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (n0 + 4 * fq + i < g.N) dst[i] = acc[t][i];
        }
      }
    }
    return;
  }
  // head mode: fused argmax over rows < V, signal rows routed to extra_out
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int v = 16 * t + fr;
    float val[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      val[i] = acc[t][i];
      if (PLANES == 2) val[i] += __shfl_xor(acc[t][i], 1, 64);
    }
    const bool owner = (v < Mv) && (PLANES == 1 || (fr & 1) == 0);
    const int m = v / PLANES;
    float bv = -INFINITY;
    int bi = INT_MAX;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n0 + 4 * fq + i;
      if (owner && n < g.N) {
        if (n < g.V) {
          if (g.logits_dbg) g.logits_dbg[static_cast<size_t>(m) * g.V + n] = val[i];
          if (val[i] > bv) { bv = val[i]; bi = n; }
        } else if (g.extra_out) {
          g.extra_out[m * g.n_extra + (n - g.V)] = val[i];
        }
      }
    }
#pragma unroll
    for (int o = 16; o < 64; o <<= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (owner && fq == 0) {
      g.part_val[static_cast<size_t>(m) * ntiles + tile] = bv;
      g.part_idx[static_cast<size_t>(m) * ntiles + tile] = bi;
    }
  }
}

__global__ __launch_bounds__(256) void k_argmax_finalize(const float* __restrict__ part_val,
                                                         const int* __restrict__ part_idx, int ntiles,
                                                         int32_t* __restrict__ argmax,
                                                         float* __restrict__ max_logit) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int m = blockIdx.x;
  float bv = -INFINITY;
  int bi = INT_MAX;
  for (int t = threadIdx.x; t < ntiles; t += 256) {
    const float v = part_val[static_cast<size_t>(m) * ntiles + t];
    const int i = part_idx[static_cast<size_t>(m) * ntiles + t];
    if (better(v, i, bv, bi)) { bv = v; bi = i; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    argmax[m] = bi;
    if (max_logit) max_logit[m] = bv;
  }
}

__global__ __launch_bounds__(256) void k_argmax_rows(const float* __restrict__ logits, int N, int V,
                                                     int n_extra, int32_t* __restrict__ argmax,
                                                     float* __restrict__ max_logit,
                                                     float* __restrict__ extra_out,
                                                     float* __restrict__ logits_dbg) {
  __shared__ float sv[4];
  __shared__ int si[4];
  const int m = blockIdx.x;
  const float* row = logits + static_cast<size_t>(m) * N;
  float bv = -INFINITY;
  int bi = INT_MAX;
  for (int n = threadIdx.x; n < V; n += 256) {
    const float v = row[n];
    if (logits_dbg) logits_dbg[static_cast<size_t>(m) * V + n] = v;
    if (better(v, n, bv, bi)) { bv = v; bi = n; }
  }
  if (extra_out && threadIdx.x < n_extra) extra_out[m * n_extra + threadIdx.x] = row[V + threadIdx.x];
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < 4; ++w)
      if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
    argmax[m] = bi;
    if (max_logit) max_logit[m] = bv;
  }
}

// Fragment layout of packed activations: for k-step s (32 values of k), column block t,
// lane (c, q) = (lane % 16, lane / 16) holds act[16 t + c][32 s + 8 q .. + 7] as bf16.
template <typename T>
__global__ __launch_bounds__(256) void k_pack_rows(const T* __restrict__ src, int M, int K, int MT,
                                                   uint4* __restrict__ apack, float* __restrict__ act) {
  const int m = blockIdx.x;
  const T* row = src + static_cast<size_t>(m) * K;
  for (int g8 = threadIdx.x; g8 < K / 8; g8 += 256) {
    float f[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = Elem<T>::load(row + g8 * 8 + e);
    if (act) {
#pragma unroll
      for (int e = 0; e < 8; ++e) act[static_cast<size_t>(m) * K + g8 * 8 + e] = f[e];
    }
    if (apack) {
      uint32_t p[4];
#pragma unroll
      for (int e = 0; e < 4; ++e)
        p[e] = static_cast<uint32_t>(f32_to_bf16(f[2 * e])) | (static_cast<uint32_t>(f32_to_bf16(f[2 * e + 1])) << 16);
      const int s = g8 >> 2, q = g8 & 3;
      apack[(static_cast<size_t>(s) * MT + (m >> 4)) * 64 + (m & 15) + 16 * q] = make_uint4(p[0], p[1], p[2], p[3]);
    }
  }
}

}  // namespace

bool gemm_mfma_supported(int M, int planes, int K) {
  const int mt = gemm_mt(M, planes);
  return (K % 128 == 0) && mt >= 1 && mt <= 9;
}

void choose_ksplit(GemmArgs& g, bool mfma) {
  if (!mfma || g.V >= 0) {
    g.ksplit = 1;
    g.kb_per_split = g.K / 128;
    return;
  }
  const int KB = g.K / 128;
  const int ntiles = gemm_ntiles(g.N);
  int want = (4096 + ntiles - 1) / ntiles;
  if (want < 1) want = 1;
  if (want > KB) want = KB;
  if (want > 32) want = 32;
  g.kb_per_split = (KB + want - 1) / want;
  g.ksplit = (KB + g.kb_per_split - 1) / g.kb_per_split;
}

hipError_t launch_gemm_valu(const GemmArgs& g, bool bf16, hipStream_t s) {
  const dim3 grid((g.N + 3) / 4);
  if (bf16)
    hipLaunchKernelGGL(k_gemv_valu<bf16_t>, grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(k_gemv_valu<float>, grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

template <int PLANES, bool HEAD>
static hipError_t launch_mfma_planes(const GemmArgs& g, hipStream_t s) {
  const int mt = gemm_mt(g.M, PLANES);
  const dim3 grid((gemm_ntiles(g.N) + 3) / 4, g.ksplit);
  const dim3 block(256);
  switch (mt) {
    case 1: hipLaunchKernelGGL((k_gemm_mfma<1, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 2: hipLaunchKernelGGL((k_gemm_mfma<2, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 3: hipLaunchKernelGGL((k_gemm_mfma<3, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 4: hipLaunchKernelGGL((k_gemm_mfma<4, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 5: hipLaunchKernelGGL((k_gemm_mfma<5, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 6: hipLaunchKernelGGL((k_gemm_mfma<6, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 7: hipLaunchKernelGGL((k_gemm_mfma<7, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 8: hipLaunchKernelGGL((k_gemm_mfma<8, PLANES, HEAD>), grid, block, 0, s, g); break;
    case 9: hipLaunchKernelGGL((k_gemm_mfma<9, PLANES, HEAD>), grid, block, 0, s, g); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s) {
  if (g.V >= 0) return g.planes == 2 ? launch_mfma_planes<2, true>(g, s) : launch_mfma_planes<1, true>(g, s);
  return g.planes == 2 ? launch_mfma_planes<2, false>(g, s) : launch_mfma_planes<1, false>(g, s);
}

hipError_t launch_argmax_finalize(const float* part_val, const int* part_idx, int ntiles, int M,
                                  int32_t* argmax, float* max_logit, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_finalize, dim3(M), dim3(256), 0, s, part_val, part_idx, ntiles, argmax, max_logit);
  return hipGetLastError();
}

hipError_t launch_argmax_rows(const float* logits, int M, int N, int V, int n_extra, int32_t* argmax,
                              float* max_logit, float* extra_out, float* logits_dbg, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_rows, dim3(M), dim3(256), 0, s, logits, N, V, n_extra, argmax, max_logit,
                     extra_out, logits_dbg);
  return hipGetLastError();
}

hipError_t launch_pack_rows(const void* src, bool bf16, int M, int K, uint4* apack, float* act,
                            hipStream_t s) {
  const int MT = gemm_mt(M, 1);
  if (bf16)
    hipLaunchKernelGGL(k_pack_rows<bf16_t>, dim3(M), dim3(256), 0, s, static_cast<const bf16_t*>(src), M, K, MT, apack, act);
  else
    hipLaunchKernelGGL(k_pack_rows<float>, dim3(M), dim3(256), 0, s, static_cast<const float*>(src), M, K, MT, apack, act);
  return hipGetLastError();
}

}  // namespace sx
