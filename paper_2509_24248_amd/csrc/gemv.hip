// Row-streaming GEMV for the draft layer's projections when the step has few rows (M <= 4,
// which is the chain-drafting case of one or a few sequences).  out[m][n] = sum_k a[m][k] w[n][k].
//
// With so few activation rows the matrix cores buy nothing: the kernel is a pure weight
// stream.  A wave takes two weight rows at a time and reads each along K with 16-byte loads,
// 1 KB per instruction and three instructions per row in flight (more waves resident beat deeper queues), multiplies with the
// fp32 activations held in LDS and reduces across its lanes.  There is no split over K, so
// nothing is left for a later kernel (or a last-arriving workgroup) to add up: the epilogue
// runs in the wave that owns the rows.  The two rows of a pair are chosen by the epilogue:
//   rows     (2p, 2p+1): residual add, fp32 / bf16 outputs, pieces of the rows' sums of
//            squares for the RMSNorm the consumer applies while staging;
//   rotary   (head*d + c, head*d + c + d/2) of the concatenated q|k|v projection: the pair
//            is rotated and stored as a query element or a cache entry (Sec. 3.1 draft layer);
//   gate     (p, I + p) of the concatenated gate|up projection: silu(gate) * up;
//   head     (2p, 2p+1) of the widened head (Eq. 1): rows below V enter a running argmax (lowest
//            index on ties) kept per wave and merged per workgroup, the signal rows V.. are
//            written out; a later launch merges the workgroups' candidates.
// Activations are staged once per workgroup as fp32, interleaved so that lane l's eight
// values of step j are two conflict-free float4 reads.
#include "common.hpp"
#include "kernels.hpp"

#include <limits.h>

namespace sx {

namespace {

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// The head's 778 MB are read once per launch and must not displace anything: non-temporal
// loads.  The layer's projections come round again one draft step later; when they fit the 256 MB
// last-level cache (228 MB at the metric's workload) ordinary loads let it keep part of them
// (measured: 764 -> 775 rounds/s; with ordinary loads in the head as well, 696).  A layer that
// does not fit is streamed like the head (ordinary loads cost 2 % there, measured on the
// matrix-core projections of the 8B- and 32B-like shapes).
template <bool STREAM>
__device__ __forceinline__ uint4 load_weights16(const char* p) {
  if constexpr (STREAM) {
    const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
  } else {
    return *reinterpret_cast<const uint4*>(p);
  }
}

__device__ __forceinline__ const char* weight_row(const GemvArgs& g, int n) {
  int s = 0, start = 0;
#pragma unroll
  for (int i = 0; i < 2; ++i)
    if (s + 1 < g.nseg && n >= g.seg_end[s]) { start = g.seg_end[s]; ++s; }
  return static_cast<const char*>(g.w[s]) + static_cast<size_t>(n - start) * g.K * 2;
}

constexpr int kHeadStepsInFlight = 2;
constexpr int kStepsInFlight = 3;   // 16-byte loads per row in flight (2 rows): few registers, more resident waves (measured best of 1..8)

// LDS position (in floats) of activation row m, element k: step j = k / 512 holds lane
// l = (k % 512) / 8's eight values as float4 [j][m][half][l]
__device__ __forceinline__ int act_pos(int M, int m, int k) {
  const int j = k >> 9, l = (k & 511) >> 3, e = k & 7;
  return (((j * M + m) * 2 + (e >> 2)) * 64 + l) * 4 + (e & 3);
}

template <int MR, int SIF, bool STREAM>
__global__ __launch_bounds__(512) void k_gemv(const GemvArgs g) {
  extern __shared__ float lds[];
  __shared__ float rs_sh[4];
  __shared__ float ssq_sh[8][4];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nwaves = blockDim.x >> 6;
  const int nt = blockDim.x;
  const int K = g.K;
  const int steps = K >> 9;             // K is a multiple of 512

  // ---- stage the activations
  if (g.a_mode == 3) {
    // 1 / rms of each row from the producer's pieces of the sum of squares
    if (wv < MR) {
      float s = 0.f;
      for (int j = lane; j < g.a_nssq; j += 64) s += g.a_ssq[wv * g.a_nssq + j];
      s = wave_sum(s);
      if (lane == 0) rs_sh[wv] = 1.0f / sqrtf(s / static_cast<float>(K) + g.a_eps);
    }
    __syncthreads();
  }
  for (int idx = threadIdx.x; idx < MR * (K >> 3); idx += nt) {
    const int m = idx / (K >> 3), k = (idx - m * (K >> 3)) << 3;
    float f[8];
    if (g.a_mode == 0 || g.a_mode == 3) {
      const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(g.a_src) + static_cast<size_t>(m) * K + k);
      const float4 x = src[0], y = src[1];
      f[0] = x.x; f[1] = x.y; f[2] = x.z; f[3] = x.w; f[4] = y.x; f[5] = y.y; f[6] = y.z; f[7] = y.w;
      if (g.a_mode == 3) {
        float gn[8];
        unpack16(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(g.a_gain) + k), gn);
        const float rs = rs_sh[m];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = f[e] * rs * gn[e];
      }
    } else if (g.a_mode == 1) {
      unpack16(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(g.a_src) + static_cast<size_t>(m) * K + k), f);
    } else {
      const int half = K >> 1;
      const bf16_t* src = k < half ? static_cast<const bf16_t*>(g.a_embed) + static_cast<size_t>(checked_token(g.a_tok[m], g.a_vocab, g.status)) * half + k
                                   : static_cast<const bf16_t*>(g.a_src) + static_cast<size_t>(m) * half + (k - half);
      unpack16(*reinterpret_cast<const uint4*>(src), f);
    }
    const int p0 = act_pos(MR, m, k);
    *reinterpret_cast<float4*>(lds + p0) = make_float4(f[0], f[1], f[2], f[3]);
    *reinterpret_cast<float4*>(lds + p0 + 256) = make_float4(f[4], f[5], f[6], f[7]);
  }
  __syncthreads();

  // ---- pairs of rows, dealt round-robin over all waves of the launch: at any time the waves read
  // one moving window of neighbouring rows (measured 0.9 % on the round against a contiguous
  // range of pairs per workgroup), and no wave gets more than one pair above the others
  const int P = (g.N + 1) >> 1;          // only the head's row count can be odd: its last pair is half empty
  float ssq[MR];
  float bestv[MR];
  int besti[MR];
#pragma unroll
  for (int m = 0; m < MR; ++m) { ssq[m] = 0.f; bestv[m] = -INFINITY; besti[m] = INT_MAX; }

  for (int p = blockIdx.x * nwaves + wv; p < P; p += gridDim.x * nwaves) {
    int n1, n2;
    if (g.epi == 1) {
      const int half = g.rope.d >> 1;
      const int head = p / half, c = p - head * half;
      n1 = head * g.rope.d + c;
      n2 = n1 + half;
    } else if (g.epi == 2) {
      n1 = p;
      n2 = P + p;
    } else {
      n1 = 2 * p;
      n2 = n1 + 1;
    }
    const char* r1 = weight_row(g, n1) + lane * 16;
    const char* r2 = weight_row(g, min(n2, g.N - 1)) + lane * 16;   // a row past the end repeats the last one, unused
    float acc1[MR], acc2[MR];
#pragma unroll
    for (int m = 0; m < MR; ++m) { acc1[m] = 0.f; acc2[m] = 0.f; }
    for (int j0 = 0; j0 < steps; j0 += SIF) {
      uint4 w1[SIF], w2[SIF];
#pragma unroll
      for (int u = 0; u < SIF; ++u) {
        const int j = j0 + u;
        const bool ok = j < steps;
        w1[u] = ok ? load_weights16<STREAM>(r1 + (static_cast<size_t>(j) << 10)) : make_uint4(0, 0, 0, 0);
        w2[u] = ok ? load_weights16<STREAM>(r2 + (static_cast<size_t>(j) << 10)) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < SIF; ++u) {
        const int j = j0 + u;
        if (j < steps) {
          float f1[8], f2[8];
          unpack16(w1[u], f1);
          unpack16(w2[u], f2);
#pragma unroll
          for (int m = 0; m < MR; ++m) {
            const float4 a0 = *reinterpret_cast<const float4*>(lds + (((j * MR + m) * 2 + 0) * 64 + lane) * 4);
            const float4 a1 = *reinterpret_cast<const float4*>(lds + (((j * MR + m) * 2 + 1) * 64 + lane) * 4);
            acc1[m] = fmaf(a0.x, f1[0], acc1[m]); acc1[m] = fmaf(a0.y, f1[1], acc1[m]);
            acc1[m] = fmaf(a0.z, f1[2], acc1[m]); acc1[m] = fmaf(a0.w, f1[3], acc1[m]);
            acc1[m] = fmaf(a1.x, f1[4], acc1[m]); acc1[m] = fmaf(a1.y, f1[5], acc1[m]);
            acc1[m] = fmaf(a1.z, f1[6], acc1[m]); acc1[m] = fmaf(a1.w, f1[7], acc1[m]);
            acc2[m] = fmaf(a0.x, f2[0], acc2[m]); acc2[m] = fmaf(a0.y, f2[1], acc2[m]);
            acc2[m] = fmaf(a0.z, f2[2], acc2[m]); acc2[m] = fmaf(a0.w, f2[3], acc2[m]);
            acc2[m] = fmaf(a1.x, f2[4], acc2[m]); acc2[m] = fmaf(a1.y, f2[5], acc2[m]);
            acc2[m] = fmaf(a1.z, f2[6], acc2[m]); acc2[m] = fmaf(a1.w, f2[7], acc2[m]);
          }
        }
      }
    }
#pragma unroll
    for (int m = 0; m < MR; ++m) {
      const float v1 = wave_sum(acc1[m]), v2 = wave_sum(acc2[m]);
      if (lane != 0) continue;
      if (g.epi == 0) {
        float x1 = v1, x2 = v2;
        if (g.residual) {
          x1 += g.residual[static_cast<size_t>(m) * g.N + n1];
          x2 += g.residual[static_cast<size_t>(m) * g.N + n2];
        }
        *reinterpret_cast<float2*>(g.out_x + static_cast<size_t>(m) * g.N + n1) = make_float2(x1, x2);
        if (g.out_store)
          *reinterpret_cast<uint32_t*>(static_cast<bf16_t*>(g.out_store) + static_cast<size_t>(m) * g.N + n1) = pack_bf16x2(x1, x2);
        ssq[m] += x1 * x1 + x2 * x2;
      } else if (g.epi == 2) {
        g.out_x[static_cast<size_t>(m) * P + p] = v1 * sigmoidf_(v1) * v2;
      } else if (g.epi == 3) {
        // rows are visited in increasing order by this wave, '>' keeps the lowest index
        if (n1 < g.V) { if (v1 > bestv[m]) { bestv[m] = v1; besti[m] = n1; } }
        else if (g.extra_out) g.extra_out[m * g.n_extra + (n1 - g.V)] = v1;
        if (n2 < g.N) {
          if (n2 < g.V) { if (v2 > bestv[m]) { bestv[m] = v2; besti[m] = n2; } }
          else if (g.extra_out) g.extra_out[m * g.n_extra + (n2 - g.V)] = v2;
        }
      } else {
        const RopeArgs& ra = g.rope;
        const int half = ra.d >> 1;
        const int hh = n1 / ra.d, c = n1 - hh * ra.d;
        const int b = m / ra.W;
        const int ps = ra.pos[b] + ra.level;
        const int slot = ra.pos[b] + (ra.node ? ra.node[m % ra.W] : 0);
        float x1 = v1, x2 = v2;
        if (hh < ra.Hq + ra.Hkv) {
          const double ang = static_cast<double>(ps) * ra.inv_freq[c];
          const double turns = rint(ang * 0.15915494309189535);
          const float red_ang = static_cast<float>(fma(-turns, 6.283185307179586, ang));
          const float cs = cosf(red_ang), sn = sinf(red_ang);
          x1 = v1 * cs - v2 * sn;
          x2 = v2 * cs + v1 * sn;
        }
        bf16_t* dst = nullptr;
        if (hh < ra.Hq) {
          dst = static_cast<bf16_t*>(ra.q_out) + (static_cast<size_t>(m) * ra.Hq + hh) * ra.d;
        } else if (slot >= 0 && slot < ra.l_max) {
          const bool is_k = hh < ra.Hq + ra.Hkv;
          const int h = is_k ? hh - ra.Hq : hh - ra.Hq - ra.Hkv;
          size_t off;
          bool ok = true;
          if (ra.paged) {
            const int page = ra.page_table[static_cast<size_t>(b) * ra.max_pages + slot / ra.page_size];
            ok = page_in_pool(page, ra.n_pages, ra.status);
            off = ((static_cast<size_t>(page) * ra.Hkv + h) * ra.page_size + slot % ra.page_size) * ra.d;
          } else {
            off = ((static_cast<size_t>(b) * ra.Hkv + h) * ra.l_max + slot) * ra.d;
          }
          if (ok) dst = static_cast<bf16_t*>(is_k ? ra.kc : ra.vc) + off;
        }
        if (dst) {
          dst[c] = f32_to_bf16(x1);
          dst[c + half] = f32_to_bf16(x2);
        }
      }
    }
  }

  // ---- head: the workgroup's best (value, index) per activation row
  if (g.epi == 3) {
    __shared__ float bv_sh[8][4];
    __shared__ int bi_sh[8][4];
    if (lane == 0) {
#pragma unroll
      for (int m = 0; m < MR; ++m) { bv_sh[wv][m] = bestv[m]; bi_sh[wv][m] = besti[m]; }
    }
    __syncthreads();
    if (threadIdx.x < MR) {
      float bv = bv_sh[0][threadIdx.x];
      int bi = bi_sh[0][threadIdx.x];
      for (int w = 1; w < nwaves; ++w)
        if (better(bv_sh[w][threadIdx.x], bi_sh[w][threadIdx.x], bv, bi)) { bv = bv_sh[w][threadIdx.x]; bi = bi_sh[w][threadIdx.x]; }
      g.part_val[threadIdx.x * gridDim.x + blockIdx.x] = bv;
      g.part_idx[threadIdx.x * gridDim.x + blockIdx.x] = bi;
    }
  }
  // ---- this workgroup's piece of the rows' sums of squares (waves added in a fixed order)
  if (g.epi == 0 && g.out_ssq) {
    if (lane == 0) {
#pragma unroll
      for (int m = 0; m < MR; ++m) ssq_sh[wv][m] = ssq[m];
    }
    __syncthreads();
    if (threadIdx.x < MR) {
      float t = 0.f;
      for (int w = 0; w < nwaves; ++w) t += ssq_sh[w][threadIdx.x];
      g.out_ssq[threadIdx.x * gridDim.x + blockIdx.x] = t;
    }
  }
}

template <int MR, int SIF, bool STREAM>
hipError_t launch_mr_sif(const GemvArgs& g, hipStream_t s) {
  const size_t lds = gemv_lds_bytes(g);
  // set once per process; a function-local static is initialised under the language's own lock,
  // so first calls from several host threads are safe
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemv<MR, SIF, STREAM>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 512);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((k_gemv<MR, SIF, STREAM>), dim3(g.grid), dim3(64 * g.waves), lds, s, g);
  return hipGetLastError();
}

// Loads per row in flight: three for the short projections, two for the head's long stream
// (measured: 1, 3, 4, 5 slower, as are grids of 1, 3, 4, .. workgroups per compute unit).
template <int MR>
hipError_t launch_mr(const GemvArgs& g, hipStream_t s) {
  if (g.epi == 3) return launch_mr_sif<MR, kHeadStepsInFlight, true>(g, s);
  return g.stream ? launch_mr_sif<MR, kStepsInFlight, true>(g, s) : launch_mr_sif<MR, kStepsInFlight, false>(g, s);
}

}  // namespace

size_t gemv_lds_bytes(const GemvArgs& g) {
  return static_cast<size_t>((g.K + 511) >> 9) * g.M * 2 * 64 * 4 * sizeof(float);
}

bool gemv_supported(int M, int N, int K) {
  GemvArgs g;
  g.M = M;
  g.K = K;
  return M >= 1 && M <= 4 && (K % 512) == 0 && N >= 2 && gemv_lds_bytes(g) <= 144 * 1024;
}

// One pair per wave at a time, eight waves per workgroup sharing one staging of the activations
// (smaller workgroups for the narrow projections were measured slower), at most three
// workgroups per compute unit.
void gemv_plan(GemvArgs& g, int num_cus, int per_cu) {
  const int P = (g.N + 1) / 2;
  g.waves = 8;
  int grid = (P + g.waves - 1) / g.waves;
  const int cap = per_cu * num_cus;
  if (grid > cap) grid = cap;
  if (grid < 1) grid = 1;
  g.grid = grid;
}

hipError_t launch_gemv(const GemvArgs& g, hipStream_t s) {
  switch (g.M) {
    case 1: return launch_mr<1>(g, s);
    case 2: return launch_mr<2>(g, s);
    case 3: return launch_mr<3>(g, s);
    case 4: return launch_mr<4>(g, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sx
