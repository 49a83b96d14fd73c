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
constexpr int kGemmWaves = 8;   // waves per workgroup, one 16-row weight tile each
constexpr int kHeadWaves = 8;    // head-mode kernels (4 and 16 waves per workgroup were measured slower, at 7 and at 56 rows)

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// The weight stream is read exactly once: non-temporal loads keep it from displacing the
// small, reused operands in L2 and measurably raise the achieved HBM rate.
__device__ __forceinline__ uint4 load_stream16(const char* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// Stage the activations of K elements [k0, k0 + kc) in LDS as MFMA operand pieces:
// entry ((s * 4 + q) * S + (v ^ gemm_lds_swizzle(q))), S = gemm_lds_row_stride(Mv), holds virtual
// row v's 8 values k0 + 32 s + 8 q .. + 7 as bf16.  Virtual row v = m * PLANES + plane: plane 0 is
// the bf16 rounding of the value, plane 1 the bf16 rounding of what that lost (fp32 activations
// keep ~16 mantissa bits).
// rs_lds (mode 3): the rows' 1 / rms, computed once per workgroup.
template <int PLANES>
__device__ __forceinline__ void stage_activations(const GemmArgs& g, uint4* a_lds, const float* rs_lds, int k0, int kc,
                                                  int nthreads) {
  const int Mvs = gemm_lds_row_stride(g.M * PLANES);
  const int groups = kc >> 3;
  for (int idx = threadIdx.x; idx < g.M * groups; idx += nthreads) {
    // four neighbouring lanes take the four 8-wide pieces of one row's 32 k (64 or 128 contiguous
    // bytes in memory), the next four lanes the next row: the LDS writes of a wave then spread
    // over the banks instead of marching down one column at the row stride
    const int sm = idx >> 2;
    const int s_ = sm / g.M, m = sm - s_ * g.M;
    const int g8 = s_ * 4 + (idx & 3);
    const int k = k0 + g8 * 8;
    uint4 hi, lo = make_uint4(0, 0, 0, 0);
    if (g.a_mode == 0 || g.a_mode == 3 || g.a_mode == 4) {
      float4 x, y;
      if (g.a_mode == 4) {
        // gate and up columns summed over the producer's slices, in slice order
        float gt[8], up[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) { gt[e] = 0.f; up[e] = 0.f; }
        const int ld = 2 * g.K;
        const float* base = static_cast<const float*>(g.a_src) + k;
        const int splanes = g.a_src_planes;
        for (int j = 0; j < g.a_nslices; ++j) {
          const size_t row = static_cast<size_t>(j / splanes) * (g.M * splanes) + m * splanes + j % splanes;
          const float4* pg = reinterpret_cast<const float4*>(base + row * ld);
          const float4* pu = reinterpret_cast<const float4*>(base + row * ld + g.K);
          const float4 a = pg[0], b = pg[1], c = pu[0], d = pu[1];
          gt[0] += a.x; gt[1] += a.y; gt[2] += a.z; gt[3] += a.w; gt[4] += b.x; gt[5] += b.y; gt[6] += b.z; gt[7] += b.w;
          up[0] += c.x; up[1] += c.y; up[2] += c.z; up[3] += c.w; up[4] += d.x; up[5] += d.y; up[6] += d.z; up[7] += d.w;
        }
        float f[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = gt[e] * sigmoidf_(gt[e]) * up[e];
        x = make_float4(f[0], f[1], f[2], f[3]);
        y = make_float4(f[4], f[5], f[6], f[7]);
      } else {
        const float4* src = reinterpret_cast<const float4*>(static_cast<const float*>(g.a_src) + static_cast<size_t>(m) * g.K + k);
        x = src[0];
        y = src[1];
        if (g.a_mode == 3) {
          float gn[8];
          unpack16(*reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(g.a_gain) + k), gn);
          const float rs = rs_lds[m];
          x.x = x.x * rs * gn[0]; x.y = x.y * rs * gn[1]; x.z = x.z * rs * gn[2]; x.w = x.w * rs * gn[3];
          y.x = y.x * rs * gn[4]; y.y = y.y * rs * gn[5]; y.z = y.z * rs * gn[6]; y.w = y.w * rs * gn[7];
        }
      }
      hi = make_uint4(pack_bf16x2(x.x, x.y), pack_bf16x2(x.z, x.w), pack_bf16x2(y.x, y.y), pack_bf16x2(y.z, y.w));
      if (PLANES == 2) {
        float f[8];
        unpack16(hi, f);
        lo = make_uint4(pack_bf16x2(x.x - f[0], x.y - f[1]), pack_bf16x2(x.z - f[2], x.w - f[3]),
                        pack_bf16x2(y.x - f[4], y.y - f[5]), pack_bf16x2(y.z - f[6], y.w - f[7]));
      }
    } else if (g.a_mode == 1) {
      hi = *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(g.a_src) + static_cast<size_t>(m) * g.K + k);
    } else {
      const int half = g.K >> 1;
      const bf16_t* src = k < half ? static_cast<const bf16_t*>(g.a_embed) + static_cast<size_t>(checked_token(g.a_tok[m], g.a_vocab, g.status)) * half + k
                                   : static_cast<const bf16_t*>(g.a_src) + static_cast<size_t>(m) * half + (k - half);
      hi = *reinterpret_cast<const uint4*>(src);
    }
    const int sw = gemm_lds_swizzle(g.M * PLANES, PLANES, g8 & 3);
    a_lds[g8 * Mvs + ((m * PLANES) ^ sw)] = hi;
    if (PLANES == 2) a_lds[g8 * Mvs + ((m * PLANES + 1) ^ sw)] = lo;
  }
}

template <int MT, int PLANES, bool HEAD>
__global__ __launch_bounds__(64 * (HEAD ? kHeadWaves : kGemmWaves))
void k_gemm_mfma(const GemmArgs g) {
  constexpr int NW = HEAD ? kHeadWaves : kGemmWaves;
  // LDS: [activation pieces of one K chunk, or two one-block buffers][per wave: one 16-row x 128-k weight tile, 4 KB]
  // weight tile entry [row][pos] holds the 16-byte piece (pos ^ row) of that row, so both the
  // coalesced writes and the per-row operand reads touch 16 distinct 16-byte slots
  extern __shared__ uint4 dyn_lds[];
  const int Mv = g.M * PLANES;
  const int Mvs = gemm_lds_row_stride(Mv);
  uint4* a_lds = dyn_lds;
  uint4* w_lds = dyn_lds + (g.kc >> 3) * Mvs;
  float* rs_lds = reinterpret_cast<float*>(w_lds + NW * 256);   // [M] 1 / rms of the rows (a_mode 3)
  if (g.a_mode == 3) {
    // one wave per row: lanes take the pieces in turn, then a fixed-order butterfly
    for (int m = threadIdx.x >> 6; m < g.M; m += NW) {
      float ssq = 0.f;
      for (int j = threadIdx.x & 63; j < g.a_nssq; j += 64) ssq += g.a_ssq[m * g.a_nssq + j];
      ssq = wave_sum(ssq);
      if ((threadIdx.x & 63) == 0) rs_lds[m] = 1.0f / sqrtf(ssq / static_cast<float>(g.K) + g.a_eps);
    }
    __syncthreads();
  }
  if (MT >= 2 && Mvs > Mv) {
    // rows Mv .. Mvs - 1 of every k piece are padding: zero once, staging never touches them
    const int pad = Mvs - Mv;
    for (int idx = threadIdx.x; idx < (g.kc >> 3) * pad; idx += 64 * NW) {
      const int g8 = idx / pad, v = Mv + idx - g8 * pad;
      a_lds[g8 * Mvs + (v ^ gemm_lds_swizzle(Mv, PLANES, g8 & 3))] = make_uint4(0, 0, 0, 0);
    }
  }
  const int lane = threadIdx.x & 63;
  const int wv = threadIdx.x >> 6;
  const int ntiles = (g.N + 15) >> 4;
  // tiles of this workgroup: NW in a row, or (plain projections spread over more workgroups) an equal share
  const bool spread = !HEAD && g.spread > 0 && g.epi == 0;
  const int t_lo = spread ? static_cast<int>(static_cast<int64_t>(blockIdx.x) * ntiles / gridDim.x) : static_cast<int>(blockIdx.x) * NW;
  const int t_hi = spread ? static_cast<int>(static_cast<int64_t>(blockIdx.x + 1) * ntiles / gridDim.x) : ntiles;
  const int tile = t_lo + wv;
  const bool active = tile < t_hi;     // waves without a tile go through the same barriers and drop the result
  const int ks = blockIdx.y;
  const int KB = g.K >> 7;
  const int kb0 = ks * g.kb_per_split;
  const int kb1 = min(KB, kb0 + g.kb_per_split);
  const int n0 = (active ? tile : ntiles - 1) << 4;
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
  const int swr = gemm_lds_swizzle(Mv, PLANES, fq);
  uint4* my = w_lds + wv * 256;

  f32x4_t acc[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) acc[t] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  // Weight blocks are requested ahead of their use into two register sets used in turn: blocks
  // kb0, kb0 + 2, .. in A, the others in B.  A set is asked for its next block as soon as its
  // tile has been written to LDS, so two blocks are in flight during the arithmetic.  The loop
  // below is written without any branch around those requests (a block index past the end asks
  // for one fixed 16-byte piece instead, and an odd block count ends with a half step whose
  // activation operands are forced to zero): a request under a branch makes the compiler merge
  // register sets after it, and the waits of those copies pull the loads back into the step that
  // issued them.  Waves that have no tile of their own (past the last tile) redo the last tile for the
  // same reason and drop the result.
  // Split projections run for a few microseconds only: their first blocks are requested before
  // the activations are staged.  A head with more than 16 activation rows (times planes) has at most
  // three workgroups per compute unit, each held up by barriers per chunk or block: requests that stay
  // in flight across those keep the memory system busy (measured at 16 fp32 rows: 272 -> 263 us).
  // Heads with fewer rows have the waves to do that without and load each block where it is used.
  constexpr bool AHEAD = !HEAD || MT >= 2;
  const int kb_last = kb1 - 1;
  uint4 wA[4], wB[4];
  const char* const spare = static_cast<const char*>(g.w[0]);   // where requests past the end are pointed
  auto request = [&](uint4 (&dst)[4], int kb) {
    const bool real = kb <= kb_last && (active || !spread);   // (a spare wave of a spread launch streams nothing)
    const size_t off = static_cast<size_t>(real ? kb : 0) << 8;
#pragma unroll
    for (int i = 0; i < 4; ++i) dst[i] = load_stream16(real ? src[i] + off : spare);
  };
  if constexpr (AHEAD) {
    request(wA, kb0);
    request(wB, kb0 + 1);
  }
  // one 128-k block: this wave's weight tile (in wr) through its private LDS tile, transposed
  // into MFMA operands, against the activation pieces at ab0 (k piece 0, row 0 of the block);
  // dead: the half step past an odd block count
  auto one_tile = [&](uint4 (&wr)[4], int kb, const uint4* ab0, bool dead) {
    if constexpr (!AHEAD) request(wr, kb);
#pragma unroll
    for (int i = 0; i < 4; ++i) my[(4 * i + (lane >> 4)) * 16 + pos] = wr[i];
    if constexpr (AHEAD) request(wr, kb + 2);
    // the tile is private to this wave, whose LDS operations retire in order: a compiler
    // fence is all that separates the writes from the transposed reads
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const uint4* ab = ab0 + fq * Mvs;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint4 wf = my[fr * 16 + ((4 * s + fq) ^ fr)];
      const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, wf);
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int v = 16 * t + fr;
        uint4 af;
        if constexpr (MT >= 2) {
          af = ab[s * 4 * Mvs + (v ^ swr)];                        // padding rows Mv.. hold zeros
        } else {
          af = ab[s * 4 * Mvs + ((v < Mvs ? v : 0) ^ swr)];
          if (v >= Mv) af = make_uint4(0, 0, 0, 0);
        }
        if (dead) af = make_uint4(0, 0, 0, 0);
        acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wa, __builtin_bit_cast(bf16x8_t, af), acc[t], 0, 0, 0);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  };

  const int kcb = g.kc >> 7;           // 128-element blocks per staged chunk
  auto half = [&](uint4 (&wr)[4], int kb) {
    const bool dead = kb >= kb1;
    const int in_chunk = (kb - kb0) % kcb;
    if (in_chunk == 0 && !dead) {
      if (kb != kb0) __syncthreads();  // everyone is done with the previous chunk
      stage_activations<PLANES>(g, a_lds, rs_lds, kb << 7, (min(kb1, kb + kcb) - kb) << 7, 64 * NW);
      __syncthreads();
    }
    one_tile(wr, kb, a_lds + in_chunk * 16 * Mvs, dead);
  };
  for (int kb = kb0; kb < kb1; kb += 2) {
    half(wA, kb);
    half(wB, kb + 1);
  }
  // (a head that reports ranked candidates merges them per workgroup below: its idle waves stay)
  if (!active && (HEAD ? g.top_b <= 1 : g.epi == 0)) return;

  // accumulator layout: lane (c = lane % 16, q = lane / 16) holds rows n0 + 4q + i of
  // activation column 16 t + c
  if (!HEAD) {
    if (active) {
#pragma unroll
      for (int t = 0; t < MT; ++t) {
        const int v = 16 * t + fr;
        if (v < Mv) {
          float* dst = g.partial + (static_cast<size_t>(ks) * Mv + v) * g.N + n0 + 4 * fq;
          if (g.epi != 0) {
            // read by another workgroup of this launch (N is a multiple of 4 here)
            if (n0 + 4 * fq < g.N) store_agent16(dst, acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
          } else if (n0 + 4 * fq + 3 < g.N && (g.N & 3) == 0) {
            *reinterpret_cast<float4*>(dst) = make_float4(acc[t][0], acc[t][1], acc[t][2], acc[t][3]);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (n0 + 4 * fq + i < g.N) dst[i] = acc[t][i];
          }
        }
      }
    }
    if (g.epi == 0) return;
    // ---- the workgroup that arrives last for this 128-row group reduces it.  The partial
    // sums are written and read at agent scope; every wave waits for its stores, the
    // workgroup meets, one thread takes a ticket, and the last workgroup reads all slices in a
    // fixed order, so the sums do not depend on who is last.
    __shared__ int s_last;
    wait_stores();
    __syncthreads();
    if (threadIdx.x == 0) {
      int last = 1;
      if (gridDim.y > 1) {
        const int ticket = atomicAdd(&g.counters[blockIdx.x], 1);
        last = ticket == static_cast<int>(gridDim.y) - 1;
        if (last) g.counters[blockIdx.x] = 0;     // everyone has arrived: ready for the next launch
      }
      s_last = last;
    }
    __syncthreads();
    if (!s_last) return;
    float4* red = reinterpret_cast<float4*>(dyn_lds);           // the tiles are done with: reuse their LDS
    float* sq_lds = reinterpret_cast<float*>(red + 64 * kGemmWaves);
    float* xs = sq_lds + 64 * kGemmWaves;                       // epi = 2: the group's finished rows [M][128]
    constexpr int NT = 64 * kGemmWaves;
    const int items = g.M * 32;                                  // float4 outputs of the group
    int lpi = 1;                                                 // threads sharing one output
    while (lpi < 16 && items * lpi * 2 <= NT) lpi <<= 1;
    const int nsl = static_cast<int>(gridDim.y) * PLANES;
    const int n0g = blockIdx.x * (16 * kGemmWaves);
    for (int base = 0; base < items; base += NT / lpi) {
      const int it = base + threadIdx.x / lpi, sub = threadIdx.x % lpi;
      const int m = it >> 5, f = it & 31;
      const int n = n0g + 4 * f;
      const bool ok = it < items && n < g.N;
      float4 a4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (ok) {
        for (int j = sub; j < nsl; j += 4 * lpi) {
          const float* src[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            const int jj = min(j + u * lpi, nsl - 1);          // past the end: a valid address, value dropped
            const size_t row = static_cast<size_t>(jj / PLANES) * Mv + m * PLANES + jj % PLANES;
            src[u] = g.partial + row * g.N + n;
          }
          float4 p4[4];
          load_agent16x4(src[0], src[1], src[2], src[3], p4);
#pragma unroll
          for (int u = 0; u < 4; ++u)
            if (j + u * lpi < nsl) { a4.x += p4[u].x; a4.y += p4[u].y; a4.z += p4[u].z; a4.w += p4[u].w; }
        }
      }
      red[threadIdx.x] = a4;
      __syncthreads();
      float sq = 0.f;
      if (ok && sub == 0) {
        float4 sum = g.residual ? *reinterpret_cast<const float4*>(g.residual + static_cast<size_t>(m) * g.N + n)
                                : make_float4(0.f, 0.f, 0.f, 0.f);
        for (int u = 0; u < lpi; ++u) {
          const float4 r4 = red[threadIdx.x + u];
          sum.x += r4.x; sum.y += r4.y; sum.z += r4.z; sum.w += r4.w;
        }
        if (g.epi == 2) *reinterpret_cast<float4*>(xs + m * 128 + 4 * f) = sum;
        else *reinterpret_cast<float4*>(g.out_x + static_cast<size_t>(m) * g.N + n) = sum;
        if (g.out_store) {
          uint2 pk;
          pk.x = pack_bf16x2(sum.x, sum.y);
          pk.y = pack_bf16x2(sum.z, sum.w);
          *reinterpret_cast<uint2*>(static_cast<bf16_t*>(g.out_store) + static_cast<size_t>(m) * g.N + n) = pk;
        }
        sq = sum.x * sum.x + sum.y * sum.y + sum.z * sum.z + sum.w * sum.w;
      }
      sq_lds[threadIdx.x] = sq;
      __syncthreads();
      if (g.out_ssq && it < items && sub == 0 && f == 0) {
        float tot = 0.f;
        for (int u = 0; u < 32; ++u) tot += sq_lds[threadIdx.x + u * lpi];
        g.out_ssq[m * static_cast<int>(gridDim.x) + blockIdx.x] = tot;
      }
      __syncthreads();
    }
    if (g.epi == 2) {
      // the group's 128 columns are whole heads of q, k or v: rotate (pairs c, c + d/2) and store
      const RopeArgs& ra = g.rope;
      const int half = ra.d >> 1;
      const int pairs = g.M * 64;                               // (row, pair) items of the group
      for (int idx = threadIdx.x; idx < pairs; idx += NT) {
        const int m = idx >> 6, pr = idx & 63;
        const int hl = pr / half, c = pr - hl * half;           // head inside the group, pair inside the head
        const int hh = n0g / ra.d + hl;                         // head among q heads, then k heads, then v heads
        if (hh >= ra.Hq + 2 * ra.Hkv) continue;
        float x1 = xs[m * 128 + hl * ra.d + c], x2 = xs[m * 128 + hl * ra.d + c + half];
        const int b = m / ra.W;
        const int ps = ra.pos[b] + ra.level;
        const int slot = ra.pos[b] + (ra.node ? ra.node[m % ra.W] : 0);
        if (hh < ra.Hq + ra.Hkv) {
          // angle in double (long positions keep their phase), reduced to [-pi, pi] in double,
          // sine and cosine of the remainder in float
          const double ang = static_cast<double>(ps) * ra.inv_freq[c];
          const double turns = rint(ang * 0.15915494309189535);
          const float red_ang = static_cast<float>(fma(-turns, 6.283185307179586, ang));
          const float cs = cosf(red_ang), sn = sinf(red_ang);
          const float r1 = x1 * cs - x2 * sn;
          const float r2 = x2 * cs + x1 * sn;
          x1 = r1;
          x2 = r2;
        }
        bf16_t* dst;
        if (hh < ra.Hq) {
          dst = static_cast<bf16_t*>(ra.q_out) + (static_cast<size_t>(m) * ra.Hq + hh) * ra.d;
        } else {
          if (slot < 0 || slot >= ra.l_max) continue;           // an entry outside the cache is not written
          const bool is_k = hh < ra.Hq + ra.Hkv;
          const int h = is_k ? hh - ra.Hq : hh - ra.Hq - ra.Hkv;
          size_t off;
          if (ra.paged) {
            const int page = ra.page_table[static_cast<size_t>(b) * ra.max_pages + slot / ra.page_size];
            if (!page_in_pool(page, ra.n_pages, ra.status)) continue;
            off = ((static_cast<size_t>(page) * ra.Hkv + h) * ra.page_size + slot % ra.page_size) * ra.d;
          } else {
            off = ((static_cast<size_t>(b) * ra.Hkv + h) * ra.l_max + slot) * ra.d;
          }
          dst = static_cast<bf16_t*>(is_k ? ra.kc : ra.vc) + off;
        }
        dst[c] = f32_to_bf16(x1);
        dst[c + half] = f32_to_bf16(x2);
      }
    }
    return;
  }
  // head mode: fused argmax (or the top_b best, best first) over rows < V of this tile,
  // signal rows routed to extra_out.  With ranked candidates (top_b > 1) the waves of the
  // workgroup first merge their tiles' lists through LDS, so the merging launch sees one list per
  // 128 weight rows instead of one per 16.
  const int TB = g.top_b > 1 ? g.top_b : 1;
  const bool merge = TB > 1;
  float* cv = reinterpret_cast<float*>(dyn_lds);              // [wave][M][TB] values, then indices
  int* ci = reinterpret_cast<int*>(cv + NW * g.M * TB);
  if (merge) __syncthreads();                                 // every wave is done with the activation pieces
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
    float cur[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int n = n0 + 4 * fq + i;
      cur[i] = -INFINITY;
      if (owner && active && n < g.N) {
        if (n < g.V) {
          if (g.logits_dbg) g.logits_dbg[static_cast<size_t>(m) * g.V + n] = val[i];
          cur[i] = val[i];
        } else if (g.extra_out) {
          g.extra_out[m * g.n_extra + (n - g.V)] = val[i];
        }
      }
    }
    for (int r = 0; r < TB; ++r) {
      float bv = -INFINITY;
      int bi = INT_MAX;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (cur[i] > bv) { bv = cur[i]; bi = n0 + 4 * fq + i; }
#pragma unroll
      for (int o = 16; o < 64; o <<= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      if (owner && fq == 0) {
        if (merge) {
          cv[(wv * g.M + m) * TB + r] = bv;
          ci[(wv * g.M + m) * TB + r] = bi;
        } else {
          g.part_val[(static_cast<size_t>(m) * ntiles + tile) * TB + r] = bv;
          g.part_idx[(static_cast<size_t>(m) * ntiles + tile) * TB + r] = bi;
        }
      }
      if (r + 1 < TB) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (n0 + 4 * fq + i == bi) cur[i] = -INFINITY;   // taken: out of the next pass
      }
    }
  }
  if (merge) {
    __syncthreads();
    // half a wave per activation row, one lane per candidate of the NW lists (at most 8 x 4):
    // pass r keeps what comes after pass r-1's pick (value descending, lower index first among
    // equals; INT_MAX marks an empty slot) and takes the best of it by a butterfly
    for (int m = 2 * wv + (lane >> 5); m < g.M; m += 2 * NW) {
      const int slot = lane & 31;
      const bool have = slot < NW * TB;
      const int w = have ? slot / TB : 0, q = have ? slot - w * TB : 0;
      const float cval = have ? cv[(w * g.M + m) * TB + q] : -INFINITY;
      const int cidx = have ? ci[(w * g.M + m) * TB + q] : INT_MAX;
      float prev_v = INFINITY;
      int prev_i = -1;
      for (int r = 0; r < TB; ++r) {
        const bool after = cval < prev_v || (cval == prev_v && cidx > prev_i);
        float bv = (cidx != INT_MAX && after) ? cval : -INFINITY;
        int bi = (cidx != INT_MAX && after) ? cidx : INT_MAX;
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) {
          const float ov = __shfl_xor(bv, o, 64);
          const int oi = __shfl_xor(bi, o, 64);
          if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        if (slot == 0) {
          g.part_val[(static_cast<size_t>(m) * gridDim.x + blockIdx.x) * TB + r] = bv;
          g.part_idx[(static_cast<size_t>(m) * gridDim.x + blockIdx.x) * TB + r] = bi;
        }
        prev_v = bv;
        prev_i = bi;
      }
    }
  }
}

constexpr int kFinalThreads = 1024;

// One block per activation row: reduce the per-tile (max, index) pairs; for the draft head
// the same block also turns the three signal logits into signals (Eqs. 3-5).
__global__ __launch_bounds__(kFinalThreads) void k_argmax_finalize(const float* __restrict__ part_val,
                                                                   const int* __restrict__ part_idx, int ntiles,
                                                                   int32_t* __restrict__ argmax,
                                                                   float* __restrict__ max_logit,
                                                                   const float* __restrict__ extra,
                                                                   int rem_activation, float* __restrict__ sig_raw,
                                                                   float* __restrict__ sig) {
  __shared__ float sv[kFinalThreads / 64];
  __shared__ int si[kFinalThreads / 64];
  const int m = blockIdx.x;
  float bv = -INFINITY;
  int bi = INT_MAX;
  constexpr int U = 10;   // candidates per thread requested at once (9497 tiles of a 151939-row head: 10)
  for (int t0 = threadIdx.x; t0 < ntiles; t0 += U * kFinalThreads) {
    float v[U];
    int i[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int t = t0 + u * kFinalThreads;
      const bool ok = t < ntiles;
      v[u] = ok ? part_val[static_cast<size_t>(m) * ntiles + t] : -INFINITY;
      i[u] = ok ? part_idx[static_cast<size_t>(m) * ntiles + t] : INT_MAX;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (better(v[u], i[u], bv, bi)) { bv = v[u]; bi = i[u]; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(bv, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
  __syncthreads();
  if (threadIdx.x < 64) {
    // the 16 waves' results, one per lane, merged by a butterfly
    const bool have = threadIdx.x < kFinalThreads / 64;
    bv = have ? sv[threadIdx.x] : -INFINITY;
    bi = have ? si[threadIdx.x] : INT_MAX;
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if (threadIdx.x == 0) {
      argmax[m] = bi;
      if (max_logit) max_logit[m] = bv;
    }
  }
  if (sig && threadIdx.x == 64) {
    const float zc = extra[m * 3 + 0], zp = extra[m * 3 + 1], zr = extra[m * 3 + 2];
    sig_raw[m * 3 + 0] = zc; sig_raw[m * 3 + 1] = zp; sig_raw[m * 3 + 2] = zr;
    sig[m * 3 + 0] = sigmoidf_(zc);
    sig[m * 3 + 1] = sigmoidf_(zp);
    sig[m * 3 + 2] = rem_activation == 0 ? fmaxf(0.f, expm1f(zr)) : (rem_activation == 1 ? sigmoidf_(zr) : zr);
  }
}

// The top_b best of each row, best first (value descending, lower index first among equals),
// from per-tile candidates (part_idx != nullptr: C = ntiles * top_b pairs, INT_MAX marks an
// empty slot) or from a full logits row (part_idx == nullptr: candidate c is (row[c], c)).
// Pass r takes the best candidate that comes after pass r-1's pick in that order.
__global__ __launch_bounds__(kFinalThreads) void k_topb_finalize(const float* __restrict__ vals,
                                                                 const int* __restrict__ idxs, int C, int stride,
                                                                 int top_b, int32_t* __restrict__ cand_tok,
                                                                 float* __restrict__ cand_logit,
                                                                 const float* __restrict__ extra, int rem_activation,
                                                                 float* __restrict__ sig_raw, float* __restrict__ sig) {
  __shared__ float sv[kFinalThreads / 64];
  __shared__ int si[kFinalThreads / 64];
  __shared__ float pick_v;
  __shared__ int pick_i;
  const int m = blockIdx.x;
  const float* rv = vals + static_cast<size_t>(m) * stride;
  const int* ri = idxs ? idxs + static_cast<size_t>(m) * stride : nullptr;
  float prev_v = INFINITY;
  int prev_i = -1;
  // candidate lists (9497 tiles x 1, or 1188 workgroups x 4 for a 151939-row head) are read once,
  // all requests at once, and the passes run from registers; a full logits row is streamed in
  // every pass.  Kept short on purpose: this kernel runs once on a cold instruction cache.
  constexpr int U = 10;
  const bool held = ri != nullptr && C <= U * kFinalThreads;
  float hv[U];
  int hi[U];
  if (held) {
    // slot groups past the end are skipped as a whole (a uniform branch); inside the last group
    // the last candidate is read again and marked empty
#pragma unroll
    for (int u = 0; u < U; ++u) {
      hv[u] = -INFINITY;
      hi[u] = INT_MAX;
      if (u * kFinalThreads < C) {
        const int c = threadIdx.x + u * kFinalThreads;
        const int cc = min(c, C - 1);
        const float v = rv[cc];
        const int i = ri[cc];
        hv[u] = v;
        hi[u] = c < C ? i : INT_MAX;
      }
    }
  }
  for (int r = 0; r < top_b; ++r) {
    float bv = -INFINITY;
    int bi = INT_MAX;
    if (held) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (u * kFinalThreads < C) {
          const bool after = (hv[u] < prev_v) | ((hv[u] == prev_v) & (hi[u] > prev_i));
          const bool take = (hi[u] != INT_MAX) & after & better(hv[u], hi[u], bv, bi);
          bv = take ? hv[u] : bv;
          bi = take ? hi[u] : bi;
        }
      }
    } else {
      for (int c = threadIdx.x; c < C; c += kFinalThreads) {
        const float v = rv[c];
        const int i = ri ? ri[c] : c;
        const bool after = v < prev_v || (v == prev_v && i > prev_i);
        if (i != INT_MAX && after && better(v, i, bv, bi)) { bv = v; bi = i; }
      }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const float ov = __shfl_xor(bv, o, 64);
      const int oi = __shfl_xor(bi, o, 64);
      if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
    __syncthreads();
    if (threadIdx.x < 64) {
      const bool have = threadIdx.x < kFinalThreads / 64;
      bv = have ? sv[threadIdx.x] : -INFINITY;
      bi = have ? si[threadIdx.x] : INT_MAX;
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int oi = __shfl_xor(bi, o, 64);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      if (threadIdx.x == 0) {
        cand_tok[m * top_b + r] = bi == INT_MAX ? -1 : bi;
        if (cand_logit) cand_logit[m * top_b + r] = bv;
        pick_v = bv;
        pick_i = bi;
      }
    }
    __syncthreads();
    prev_v = pick_v;
    prev_i = pick_i;
  }
  if (sig && threadIdx.x == 64) {
    const float zc = extra[m * 3 + 0], zp = extra[m * 3 + 1], zr = extra[m * 3 + 2];
    sig_raw[m * 3 + 0] = zc; sig_raw[m * 3 + 1] = zp; sig_raw[m * 3 + 2] = zr;
    sig[m * 3 + 0] = sigmoidf_(zc);
    sig[m * 3 + 1] = sigmoidf_(zp);
    sig[m * 3 + 2] = rem_activation == 0 ? fmaxf(0.f, expm1f(zr)) : (rem_activation == 1 ? sigmoidf_(zr) : zr);
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
  if (extra_out && static_cast<int>(threadIdx.x) < n_extra) extra_out[m * n_extra + threadIdx.x] = row[V + threadIdx.x];
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

template <typename T>
__global__ __launch_bounds__(256) void k_unpack_rows(const T* __restrict__ src, int K, float* __restrict__ act) {
  const int m = blockIdx.x;
  for (int k = threadIdx.x; k < K; k += 256)
    act[static_cast<size_t>(m) * K + k] = Elem<T>::load(src + static_cast<size_t>(m) * K + k);
}

}  // namespace

bool gemm_mfma_supported(int M, int planes, int K) {
  const int mt = gemm_mt(M, planes);
  return (K % 128 == 0) && mt >= 1 && mt <= 9;
}

// Split projections: workgroups that share a compute unit, and the most K ranges (measured at the
// 32B-like shapes with 16 rows and the 8B-like ones with 8: three per unit 10 % slower on the
// step's projections, up to 24 ranges the same, at most 8 ranges 5 % slower).
constexpr int kGemmPerCu = 2, kGemmMaxKsplit = 16;

void choose_ksplit(GemmArgs& g, bool mfma, int num_cus) {
  const int KB = g.K / 128;
  if (!mfma) {
    g.ksplit = 1;
    g.kb_per_split = KB;
    g.kc = g.K;
    return;
  }
  const int Mv = g.M * g.planes;
  const int Mvs = gemm_lds_row_stride(Mv);
  const int block_bytes = Mvs * 128 * 2;       // LDS bytes of one 128-k block of activation pieces
  int budget;
  if (g.V >= 0) {
    g.ksplit = 1;
    g.kb_per_split = KB;
    // head-mode kernels run for 100+ us: a smaller activation chunk lets three workgroups share a
    // compute unit, which is worth more than the extra chunk barriers (measured at M = 8, 56, 64)
    budget = (Mv > 32 ? 32 : 20) * 1024;
  } else {
    // The projections run for some tens of microseconds, so what counts is that all their
    // workgroups are resident at once and keep enough loads in flight: kGemmPerCu workgroups
    // share a compute unit (the activation chunk is sized so that their LDS fits), and K is
    // split until the 128-row groups times the K ranges fill those places.  (One workgroup of
    // 96 KB per compute unit left the gate/up, q/k/v and down projections of the 32B-like shapes
    // with 280-400 workgroups for 256 places: a second, nearly empty round.)
    const int groups = gemm_groups(g.N);
    const int places = kGemmPerCu * num_cus;
    int want = places / groups;
    if (want > kGemmMaxKsplit) want = kGemmMaxKsplit;
    if (want > KB) want = KB;
    if (want < 1) want = 1;
    g.kb_per_split = (KB + want - 1) / want;
    g.ksplit = (KB + g.kb_per_split - 1) / g.kb_per_split;
    budget = (160 * 1024 - 1024) / kGemmPerCu - kGemmWaves * 4096 - 2048;
    // One K range and between half and all of the places taken (the gate/up projection of the 32B-like
    // shapes: 400 groups for 512 places): compute units with two workgroups then set the time while the
    // others idle.  The tiles are dealt to all places in equal shares instead (6.25 tiles each there).
    const int ntiles = gemm_ntiles(g.N);
    g.spread = (g.ksplit == 1 && groups < places && ntiles >= 4 * places) ? places : 0;
  }
  // activations staged in LDS per chunk: the whole K range if it fits the budget
  int kcb = budget / block_bytes;
  if (kcb < 1) kcb = 1;
  if (kcb > g.kb_per_split) kcb = g.kb_per_split;
  g.kc = kcb * 128;
  // the LM head over more than 32 rows has a kernel of its own
  head_wide_plan(g, num_cus);
}

__global__ void k_zero_i32(int* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

hipError_t launch_zero_i32(int* p, int n, hipStream_t s) {
  hipLaunchKernelGGL(k_zero_i32, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

hipError_t launch_gemm_valu(const GemmArgs& g, bool bf16, hipStream_t s) {
  const dim3 grid((g.N + 3) / 4);
  if (bf16)
    hipLaunchKernelGGL(k_gemv_valu<bf16_t>, grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(k_gemv_valu<float>, grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

size_t gemm_mfma_lds_bytes(const GemmArgs& g) {
  // activation pieces, one weight tile per wave, the rows' 1 / rms; the reducing epilogue
  // overlays 512 float4 + 512 float on the front
  const size_t main = (static_cast<size_t>(g.kc >> 3) * gemm_lds_row_stride(g.M * g.planes) + static_cast<size_t>(g.V >= 0 ? kHeadWaves : kGemmWaves) * 256) * 16 +
                      ((static_cast<size_t>(g.M) * sizeof(float) + 15) & ~static_cast<size_t>(15));
  const size_t overlay = g.epi == 0 ? 0 : static_cast<size_t>(64 * kGemmWaves) * 20 + (g.epi == 2 ? static_cast<size_t>(g.M) * 512 : 0);
  return main > overlay ? main : overlay;
}

template <int MT, int PLANES, bool HEAD>
static hipError_t launch_one(const GemmArgs& g, hipStream_t s) {
  // set once per process; a function-local static is initialised under the language's own lock,
  // so first calls from several host threads are safe
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_mfma<MT, PLANES, HEAD>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 256);
  if (attr != hipSuccess) return attr;
  constexpr int NW = HEAD ? kHeadWaves : kGemmWaves;
  const bool spread = !HEAD && g.spread > 0 && g.epi == 0 && g.ksplit == 1;
  const dim3 grid(spread ? g.spread : (gemm_ntiles(g.N) + NW - 1) / NW, g.ksplit);
  hipLaunchKernelGGL((k_gemm_mfma<MT, PLANES, HEAD>), grid, dim3(64 * NW), gemm_mfma_lds_bytes(g), s, g);
  return hipGetLastError();
}

template <int PLANES, bool HEAD>
static hipError_t launch_mfma_planes(const GemmArgs& g, hipStream_t s) {
  switch (gemm_mt(g.M, PLANES)) {
    case 1: return launch_one<1, PLANES, HEAD>(g, s);
    case 2: return launch_one<2, PLANES, HEAD>(g, s);
    case 3: return launch_one<3, PLANES, HEAD>(g, s);
    case 4: return launch_one<4, PLANES, HEAD>(g, s);
    case 5: return launch_one<5, PLANES, HEAD>(g, s);
    case 6: return launch_one<6, PLANES, HEAD>(g, s);
    case 7: return launch_one<7, PLANES, HEAD>(g, s);
    case 8: return launch_one<8, PLANES, HEAD>(g, s);
    case 9: return launch_one<9, PLANES, HEAD>(g, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_gemm_mfma(const GemmArgs& g, hipStream_t s) {
  if (g.wide) return launch_head_wide(g, s);
  if (g.V >= 0) return g.planes == 2 ? launch_mfma_planes<2, true>(g, s) : launch_mfma_planes<1, true>(g, s);
  return g.planes == 2 ? launch_mfma_planes<2, false>(g, s) : launch_mfma_planes<1, false>(g, s);
}

hipError_t launch_argmax_finalize(const float* part_val, const int* part_idx, int ntiles, int M,
                                  int32_t* argmax, float* max_logit, hipStream_t s, const float* extra,
                                  int rem_activation, float* sig_raw, float* sig) {
  hipLaunchKernelGGL(k_argmax_finalize, dim3(M), dim3(kFinalThreads), 0, s, part_val, part_idx, ntiles, argmax,
                     max_logit, extra, rem_activation, sig_raw, sig);
  return hipGetLastError();
}

hipError_t launch_topb_finalize(const float* vals, const int* idxs, int C, int stride, int top_b, int M,
                                int32_t* cand_tok, float* cand_logit, hipStream_t s, const float* extra,
                                int rem_activation, float* sig_raw, float* sig) {
  hipLaunchKernelGGL(k_topb_finalize, dim3(M), dim3(kFinalThreads), 0, s, vals, idxs, C, stride, top_b, cand_tok,
                     cand_logit, extra, rem_activation, sig_raw, sig);
  return hipGetLastError();
}

hipError_t launch_argmax_rows(const float* logits, int M, int N, int V, int n_extra, int32_t* argmax,
                              float* max_logit, float* extra_out, float* logits_dbg, hipStream_t s) {
  hipLaunchKernelGGL(k_argmax_rows, dim3(M), dim3(256), 0, s, logits, N, V, n_extra, argmax, max_logit,
                     extra_out, logits_dbg);
  return hipGetLastError();
}

hipError_t launch_unpack_rows(const void* src, bool bf16, int M, int K, float* act, hipStream_t s) {
  if (bf16)
    hipLaunchKernelGGL(k_unpack_rows<bf16_t>, dim3(M), dim3(256), 0, s, static_cast<const bf16_t*>(src), K, act);
  else
    hipLaunchKernelGGL(k_unpack_rows<float>, dim3(M), dim3(256), 0, s, static_cast<const float*>(src), K, act);
  return hipGetLastError();
}

}  // namespace sx
