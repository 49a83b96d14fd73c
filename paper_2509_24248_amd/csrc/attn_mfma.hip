// bf16 verification attention on the matrix cores (head_dim 128), HBM-bound by design.
//
// Work split: grid = (KV chunks, KV heads, sequences); a workgroup of four waves owns one
// chunk of one (sequence, KV head) and all R = G * n_q query rows that share that head.
// Each wave walks its own 32-key tiles of the chunk with an online softmax of its own, so
// the waves never wait for each other inside the loop; they merge once at the end.
//
// Per tile, with S^T = K Q^T and O^T = V^T P^T (the transposed forms keep the softmax row
// on a fixed lane and let P stay in registers between the two products):
//   K rows arrive as coalesced 256-byte segments, go through a swizzled LDS tile and are
//   read back as MFMA A operands (row = key, 8 consecutive d per lane);
//   V rows are written to LDS transposed ([d][key], keys in the order the P^T operand
//   uses), so the A operand of the second product is again a plain row read;
//   Q^T operand pieces (B operands) stay in registers for the whole kernel.
// The next tile's K/V are already in flight (registers) while the current one is used.
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

constexpr int kAW = 4;                 // waves per workgroup
constexpr int kVRow = 72;              // bytes per V^T row in LDS: 32 keys * 2 B + 8 B pad
constexpr int kKTile = 32 * 256;       // bytes of one wave's K tile
constexpr int kVTile = 128 * kVRow;    // bytes of one wave's V^T tile
constexpr int kORow = 132;             // floats per row of the merge buffer (128 + pad)

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint4 ld_stream16(const char* p) {
  const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}

// key handled by load instruction i (0..7) of lane group u = lane / 16: consecutive
// instructions of a lane fetch keys 2m and 2m+1, which sit next to each other in a V^T row
__device__ __forceinline__ int tile_key(int i, int u) { return 2 * (4 * (i >> 1) + u) + (i & 1); }

// position of a tile key inside a V^T row = its slot in the P^T operand: lane group q holds
// keys 4q..4q+3 of the first 16-key half, then keys 4q..4q+3 of the second half
__device__ __forceinline__ int vt_pos(int key) { return ((key & 12) << 1) | ((key >> 4) << 2) | (key & 3); }

// NG = 1: the four waves split the chunk's key tiles four ways and each handles all rows
// (R <= 64).  NG = 2: two row groups of up to 64 rows; the two waves of a group split the
// key tiles two ways (each tile is then fetched by one wave of either group: the second
// fetch is served by the cache, HBM still sees it once).
template <int RT, int NG, bool PAGED>
__global__ __launch_bounds__(64 * kAW) void k_attn_mfma(const AttnArgs a) {
  constexpr int KW = kAW / NG;          // waves sharing a row group = ways the keys are split
  extern __shared__ uint4 smem4[];
  char* smem = reinterpret_cast<char*>(smem4);
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int split = blockIdx.x, g = blockIdx.y, b = blockIdx.z;
  const int G = a.Hq / a.Hkv;
  const int R = G * a.n_q;
  const int L = a.ctx_len[b];
  const int total = L + a.n_q;
  const int s0 = split * a.chunk;
  if (s0 >= total) return;  // the whole workgroup leaves together
  const int s1 = min(total, s0 + a.chunk);
  const int fr = lane & 15, fq = lane >> 4;
  const int rg = wv / KW, kw = wv % KW;
  const int row0 = rg * 16 * RT;        // first query row of this wave's group

  char* k_lds = smem + wv * (kKTile + kVTile);
  char* v_lds = k_lds + kKTile;

  // ---- Q^T operand pieces and per-row mask words
  uint4 qf[4][RT];
  uint64_t rowmask[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int rho = row0 + 16 * t + fr;
    const bool valid = rho < R;
    const int i = valid ? rho / G : 0;
    const int hh = valid ? rho - i * G : 0;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q) + ((static_cast<size_t>(b) * a.n_q + i) * a.Hq + g * G + hh) * 128 + fq * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      qf[ks][t] = valid ? *reinterpret_cast<const uint4*>(qp + ks * 32) : make_uint4(0, 0, 0, 0);
    rowmask[t] = !valid ? 0ull : (a.mask ? a.mask[static_cast<size_t>(b) * a.n_q + i] : ((2ull << i) - 1ull));
  }

  f32x4_t oacc[8][RT];
  float m_run[RT], l_run[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) oacc[dt][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  const float sl2 = a.scale * 1.44269504088896340736f;  // scores are kept in log2 units

  // Addresses: a 64-bit base per (sequence, head) or per page, plus 32-bit offsets.  A tile is
  // 32 keys starting at a multiple of 32, so with pages of 16 * 2^n tokens it touches at most
  // two pages: the one of key 0 and the one of key 16.  Their ids are fetched one tile ahead
  // of the K/V loads that need them, so no load ever waits on a page-table read.
  const int ps_shift = 31 - __builtin_clz(a.page_size);
  const char* kbase = static_cast<const char*>(a.k);
  const char* vbase = static_cast<const char*>(a.v);
  const uint32_t lane_off = (lane & 15) << 4;
  size_t seq_row = 0;
  const int32_t* ptab = nullptr;
  if (PAGED) {
    ptab = a.page_table + static_cast<size_t>(b) * a.max_pages;
  } else {
    seq_row = (static_cast<size_t>(b) * a.Hkv + g) * a.l_max;
  }
  int pg_a = 0, pg_b = 0;   // page ids of the tile whose K/V are fetched next
  auto fetch_pages = [&](int t0) {
    if (PAGED) {
      pg_a = ptab[t0 >> ps_shift];
      pg_b = ptab[min(t0 + 16, s1 - 1) >> ps_shift];
    }
  };

  uint4 kreg[8], vreg[8];
  auto fetch = [&](int t0) {
    size_t row_a, row_b = 0;
    if (PAGED) {
      row_a = (static_cast<size_t>(pg_a) * a.Hkv + g) * a.page_size;
      row_b = (static_cast<size_t>(pg_b) * a.Hkv + g) * a.page_size;
    } else {
      row_a = seq_row + t0;
    }
    const int page0 = t0 >> ps_shift;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int p = min(t0 + tile_key(i, fq), s1 - 1);  // keys past the range are masked below
      size_t off;
      if (PAGED) {
        const size_t row = ((p >> ps_shift) == page0 ? row_a : row_b) + (p & (a.page_size - 1));
        off = row * 256 + lane_off;
      } else {
        off = (row_a + static_cast<uint32_t>(p - t0)) * 256 + lane_off;
      }
      kreg[i] = ld_stream16(kbase + off);
      vreg[i] = ld_stream16(vbase + off);
    }
  };

  int t0 = s0 + 32 * kw;
  if (t0 < s1) {
    fetch_pages(t0);
    fetch(t0);
    if (t0 + 32 * KW < s1) fetch_pages(t0 + 32 * KW);
  }
  for (; t0 < s1; t0 += 32 * KW) {
    // ---- registers -> LDS: K swizzled rows, V transposed
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int key = tile_key(i, fq);
      reinterpret_cast<uint4*>(k_lds)[key * 16 + ((lane & 15) ^ (key & 15))] = kreg[i];
    }
#pragma unroll
    for (int i2 = 0; i2 < 4; ++i2) {
      const int pos = vt_pos(tile_key(2 * i2, fq));  // even; the odd key of the pair follows it
      const uint4 va = vreg[2 * i2], vb = vreg[2 * i2 + 1];
      const uint32_t wa[4] = {va.x, va.y, va.z, va.w}, wb[4] = {vb.x, vb.y, vb.z, vb.w};
      char* base = v_lds + ((lane & 15) * 8) * kVRow + pos * 2;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        *reinterpret_cast<uint32_t*>(base + (2 * e) * kVRow) = (wa[e] & 0xFFFFu) | (wb[e] << 16);
        *reinterpret_cast<uint32_t*>(base + (2 * e + 1) * kVRow) = (wa[e] >> 16) | (wb[e] & 0xFFFF0000u);
      }
    }
    const int tnext = t0 + 32 * KW;
    if (tnext < s1) {
      fetch(tnext);                                         // page ids arrived during the last tile
      if (tnext + 32 * KW < s1) fetch_pages(tnext + 32 * KW);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // ---- S^T = K Q^T for the two 16-key halves
    f32x4_t sacc[2][RT];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < RT; ++t) sacc[j][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const uint4 kf = reinterpret_cast<const uint4*>(k_lds)[(16 * j + fr) * 16 + ((4 * ks + fq) ^ fr)];
        const bf16x8_t ka = __builtin_bit_cast(bf16x8_t, kf);
#pragma unroll
        for (int t = 0; t < RT; ++t)
          sacc[j][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, __builtin_bit_cast(bf16x8_t, qf[ks][t]), sacc[j][t], 0, 0, 0);
      }

    // ---- online softmax; lane (row, q) owns keys t0 + 16 j + 4 q + e of its row
    const bool need_mask = t0 + 32 > min(L, s1);
    uint4 pf[RT];
    bool rescale = false;
    float alpha[RT];
#pragma unroll
    for (int t = 0; t < RT; ++t) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float v = sacc[j][t][e] * sl2;
          if (need_mask) {
            const int p = t0 + 16 * j + 4 * fq + e;
            bool vis = p < s1;
            if (vis && p >= L) vis = (rowmask[t] >> (p - L)) & 1ull;
            if (!vis) v = -INFINITY;
          }
          x[4 * j + e] = v;
        }
      float mt = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      mt = fmaxf(mt, __shfl_xor(mt, 16, 64));
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
      const float m_new = fmaxf(m_run[t], mt);
      float al = 1.f;
      float pr[8];
      if (m_new == -INFINITY) {
#pragma unroll
        for (int e = 0; e < 8; ++e) pr[e] = 0.f;
      } else {
        al = __builtin_amdgcn_exp2f(m_run[t] - m_new);
#pragma unroll
        for (int e = 0; e < 8; ++e) pr[e] = __builtin_amdgcn_exp2f(x[e] - m_new);
      }
      pf[t] = make_uint4(pack_bf16x2(pr[0], pr[1]), pack_bf16x2(pr[2], pr[3]), pack_bf16x2(pr[4], pr[5]), pack_bf16x2(pr[6], pr[7]));
      l_run[t] = l_run[t] * al + (((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7])));
      m_run[t] = m_new;
      alpha[t] = al;
      rescale = rescale || (al != 1.f);
    }
    if (__builtin_amdgcn_ballot_w64(rescale) != 0ull) {
#pragma unroll
      for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          oacc[dt][t][0] *= alpha[t]; oacc[dt][t][1] *= alpha[t];
          oacc[dt][t][2] *= alpha[t]; oacc[dt][t][3] *= alpha[t];
        }
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      const uint2* vp = reinterpret_cast<const uint2*>(v_lds + (16 * dt + fr) * kVRow + fq * 16);
      const uint2 v0 = vp[0], v1 = vp[1];
      const bf16x8_t va = __builtin_bit_cast(bf16x8_t, make_uint4(v0.x, v0.y, v1.x, v1.y));
#pragma unroll
      for (int t = 0; t < RT; ++t)
        oacc[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, __builtin_bit_cast(bf16x8_t, pf[t]), oacc[dt][t], 0, 0, 0);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
  }

  // ---- merge the waves of each row group (fixed order), then one partial per workgroup
  float* ml_lds = reinterpret_cast<float*>(smem + kAW * (kKTile + kVTile));  // [kAW][16 RT][2]
  float* o_lds = reinterpret_cast<float*>(smem);                            // [NG 16 RT][kORow], overlays the tiles
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    l_run[t] = l;
    if (fq == 0) {
      ml_lds[(wv * 16 * RT + 16 * t + fr) * 2 + 0] = m_run[t];
      ml_lds[(wv * 16 * RT + 16 * t + fr) * 2 + 1] = l;
    }
  }
  __syncthreads();
  const size_t unit = (static_cast<size_t>(b) * a.Hkv + g) * a.nsplit + split;
  float fself[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    float mm = -INFINITY;
#pragma unroll
    for (int ww = 0; ww < KW; ++ww) mm = fmaxf(mm, ml_lds[((rg * KW + ww) * 16 * RT + 16 * t + fr) * 2]);
    float lt = 0.f;
    fself[t] = 0.f;
#pragma unroll
    for (int ww = 0; ww < KW; ++ww) {
      const float mw = ml_lds[((rg * KW + ww) * 16 * RT + 16 * t + fr) * 2];
      const float fw = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm);
      lt = fmaf(fw, ml_lds[((rg * KW + ww) * 16 * RT + 16 * t + fr) * 2 + 1], lt);
      if (ww == kw) fself[t] = fw;
    }
    const int rho = row0 + 16 * t + fr;
    if (kw == 0 && fq == 0 && rho < R) {
      a.part_ml[(unit * R + rho) * 2 + 0] = mm;
      a.part_ml[(unit * R + rho) * 2 + 1] = lt;
    }
  }
  for (int ww = 0; ww < KW; ++ww) {
    if (kw == ww) {
#pragma unroll
      for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          float4* dst = reinterpret_cast<float4*>(o_lds + (row0 + 16 * t + fr) * kORow + 16 * dt + 4 * fq);
          float4 v = make_float4(oacc[dt][t][0] * fself[t], oacc[dt][t][1] * fself[t],
                                 oacc[dt][t][2] * fself[t], oacc[dt][t][3] * fself[t]);
          if (ww != 0) {
            const float4 o = *dst;
            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
          }
          *dst = v;
        }
    }
    __syncthreads();
  }
  for (int idx = threadIdx.x; idx < R * 32; idx += 64 * kAW) {
    const int r = idx >> 5, c4 = idx & 31;
    *reinterpret_cast<float4*>(a.part_o + (unit * R + r) * 128 + c4 * 4) =
        *reinterpret_cast<const float4*>(o_lds + r * kORow + c4 * 4);
  }
}

size_t mfma_smem_bytes(int RT, int NG) {
  const size_t tiles = static_cast<size_t>(kAW) * (kKTile + kVTile);
  const size_t obuf = static_cast<size_t>(16) * RT * NG * kORow * sizeof(float);  // <= tiles for RT * NG <= 8
  (void)obuf;
  return tiles + static_cast<size_t>(kAW) * 16 * RT * 2 * sizeof(float);
}

template <int RT, int NG, bool PAGED>
hipError_t launch_one(const AttnArgs& a, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_mfma<RT, NG, PAGED>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((k_attn_mfma<RT, NG, PAGED>), dim3(a.nsplit, a.Hkv, a.B), dim3(64 * kAW), mfma_smem_bytes(RT, NG), s, a);
  return hipGetLastError();
}

template <int RT, int NG>
hipError_t launch_rt(const AttnArgs& a, hipStream_t s) {
  return a.paged ? launch_one<RT, NG, true>(a, s) : launch_one<RT, NG, false>(a, s);
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
  const int R = (a.Hq / a.Hkv) * a.n_q;
  const bool pow2 = (a.page_size & (a.page_size - 1)) == 0;
  return a.dtype == 1 && a.d == 128 && R <= 128 && (!a.paged || (pow2 && a.page_size >= 16));
}

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s) {
  const int R = (a.Hq / a.Hkv) * a.n_q;
  if (R <= 64) {
    switch ((R + 15) / 16) {
      case 1: return launch_rt<1, 1>(a, s);
      case 2: return launch_rt<2, 1>(a, s);
      case 3: return launch_rt<3, 1>(a, s);
      default: return launch_rt<4, 1>(a, s);
    }
  }
  switch ((R + 31) / 32) {   // row tiles per group, two groups
    case 3: return launch_rt<3, 2>(a, s);
    default: return launch_rt<4, 2>(a, s);
  }
}

}  // namespace sx
