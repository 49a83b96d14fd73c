// bf16 verification attention on the matrix cores (head_dim 128), HBM-bound by design.
//
// A workgroup takes an equal share of all keys of the launch (attn_sched.hpp): one or more
// segments, each a key range of one (sequence, KV head) unit, processed against all
// R = G * n_q query rows that share that head, so the cache is read once.
//
// Inside a workgroup there are two independent tile rings (key groups); ring kg takes the
// 32-key tiles kg, kg+2, ... of the chunk.  A ring is S slots of 16 KB in LDS (K tile + V
// tile).  Tiles are brought in by direct global->LDS loads (16 bytes per lane, streaming),
// issued S-1 tiles ahead by the ring's waves in turn, so most of the LDS holds bytes in
// flight.  Each of the ring's NR waves owns one 16-row tile of the queries and computes it
// against every tile of the ring:
//   S^T = K Q^T : A operand = K rows (row = key, 8 consecutive d per lane) read from the
//                 XOR-swizzled K tile; B operand = Q^T pieces held in registers;
//   softmax     : online, per wave, in log2 units; lane (row, q) owns 8 keys of its row;
//   O^T += V^T P^T : A operand = V^T read from the row-major V tile with the LDS transpose
//                 load (ds_read_b64_tr_b16), B operand = P^T straight from the softmax
//                 registers.
// One workgroup barrier per tile step hands a landed tile to the waves and frees the slot
// consumed one step earlier.  The two rings merge at the end in a fixed order.
#include "attn_sched.hpp"
#include "common.hpp"
#include "kernels.hpp"

namespace sx {

namespace {

constexpr int kNK = 2;                 // tile rings (key groups) per workgroup
constexpr int kSlot = 16384;           // bytes of one ring slot: K tile then V tile
constexpr int kORow = 132;             // floats per row of the merge buffer (128 + pad)
// From kBigFrom waves per ring (more than 48 query rows per KV head) one workgroup is resident per
// compute unit (its eight to sixteen waves need more than the 96-128 registers per lane that two
// workgroups would leave them) and its rings take kBigStages slots; below that, two workgroups of
// two-slot rings.  Measured at 64 / 72 rows per KV head (8B-like tree block / 32B-like chain block):
// two resident workgroups with spills 41.6 us against 31.3 us with one; two, three and four slots
// within 3 % of each other at 72 rows.
constexpr int kBigFrom = 4, kBigStages = 4;
// K operand reads / V operand read pairs issued ahead of the matrix instructions that use them: as
// many as the registers allow (one resident workgroup: all eight K reads, four V pairs)
constexpr int k_ahead(int nr) { return nr >= kBigFrom ? 8 : 4; }
constexpr int v_ahead(int nr) { return nr >= kBigFrom ? 4 : 3; }
constexpr int kMaxChunkPages = 2048;   // page ids of one chunk kept in LDS (8 KB)

typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr_t;
typedef const __attribute__((address_space(1))) void* glb_ptr_t;

// XOR swizzle of the 16-byte chunks of a tile row.  K rows are read one row per lane (16 rows
// at once): chunk ^ (key % 16) spreads them over all banks.  V rows are read by the transpose
// load, 4 rows x 2 adjacent chunks at once: chunk ^ (2 (key % 8)) keeps those eight apart.
__device__ __forceinline__ int swz_k(int key) { return key & 15; }
__device__ __forceinline__ int swz_v(int key) { return (key & 7) << 1; }

// s_waitcnt immediate that waits for vmcnt <= n only (gfx9 encoding: vmcnt in bits 3:0 and
// 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima)
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | (((n >> 4) & 3) << 14); }

// Direct global -> LDS load, 16 bytes per lane: lane l's bytes land at lds_base + 16 l
// (lds_base wave-uniform).  Written as an instruction rather than through the builtin so that
// the compiler does not put a full vector-memory wait in front of every later LDS read; the
// kernel paces these loads itself with s_waitcnt vmcnt and a barrier.  "nt" marks the stream
// as read-once.  m0 is written here and used by nothing else in these kernels.
// Same with a wave-uniform 64-bit base and a 32-bit per-lane byte offset.
__device__ __forceinline__ void load_to_lds16(const void* base, uint32_t off, const void* lds_base) {
  const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)lds_base));
  const uint64_t b64 = reinterpret_cast<uint64_t>(base);   // uniform by construction: pin it to scalar registers
  // (readfirstlane returns a signed int: go through uint32_t so the low half is not sign-extended)
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(b64))));
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(static_cast<uint32_t>(b64 >> 32))));
  const uint64_t sb = static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32);
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(l), "v"(off), "s"(sb) : "memory");
}

__device__ __forceinline__ void load_to_lds16(const void* src, const void* lds_base) {
  const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)lds_base));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(l), "v"(src) : "memory");
}

// LDS words of the schedule's prefix table (B + 1 entries, rounded to 16 bytes)
__host__ __device__ constexpr int sched_words(int B) { return (B + 1 + 3) & ~3; }

constexpr int front_bytes(int rp, int stages) {
  return kNK * stages * kSlot > rp * kORow * 4 ? kNK * stages * kSlot : rp * kORow * 4;
}

// waves per SIMD the register allocation has to leave room for: the resident workgroups' waves on
// four SIMDs
constexpr int min_waves_per_simd(int nr) { return ((nr < kBigFrom ? 2 : 1) * kNK * nr + 3) / 4; }

// NR waves per ring, each owning RTW 16-row tiles of the queries (rows 16 (rr RTW + t) ..).
// RTW = 2 halves the LDS reads per query row (K and V operands are fetched once per wave and
// used for both row tiles) at the price of fewer, fatter waves; measured slower than RTW = 1
// at R = 72, so the launcher below uses one row tile per wave throughout.
template <int NR, int RTW, int S, bool PAGED>
__global__ __launch_bounds__(64 * kNK * NR, min_waves_per_simd(NR)) void k_attn_ring(const AttnArgs a) {
  constexpr int RP = 16 * NR * RTW;             // query rows covered (padded)
  constexpr int kKAhead = k_ahead(NR), kVAhead = v_ahead(NR);
  // LDS: [ring 0: S slots][ring 1: S slots] (later overlaid by the merge buffer [RP][kORow]),
  // then the (max, sum) table for the merge, the schedule's prefix table, the page ids of the segment
  constexpr int kFront = front_bytes(RP, S);
  extern __shared__ uint4 smem4[];
  char* smem = reinterpret_cast<char*>(smem4);
  float* ml_lds = reinterpret_cast<float*>(smem + kFront);
  int* sched_lds = reinterpret_cast<int*>(smem + kFront + kNK * RP * 2 * sizeof(float));
  int* pg_lds = sched_lds + sched_words(a.B);
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int kg = wv / NR, rr = wv % NR;
  const int G = a.Hq / a.Hkv;
  const int R = G * a.n_q;
  attn_sched_build(a, sched_lds);
  const int T = a.Hkv * sched_lds[a.B];
  const int W = attn_sched_workgroups(T, a.wgrid);
  if (blockIdx.x == 0) {
    // the merging kernel reads the split back from here
    for (int i = threadIdx.x; i <= a.B; i += 64 * kNK * NR) a.sched[i] = sched_lds[i];
    if (threadIdx.x == 0) a.sched[a.B + 1] = W;
  }
  if (static_cast<int>(blockIdx.x) >= W) return;  // the whole workgroup leaves together
  const int x_hi = attn_sched_lo(blockIdx.x + 1, T, W);
  for (int x_cur = attn_sched_lo(blockIdx.x, T, W); x_cur < x_hi;) {
  const AttnSeg seg = attn_sched_segment(a, sched_lds, x_cur, x_hi);
  x_cur = seg.next;
  const int g = seg.g, b = seg.b;
  const int L = seg.L;
  const int s0 = seg.s0, s1 = seg.s1;
  const int ntl = (s1 - s0 + 31) >> 5;          // 32-key tiles in this segment
  const int nit = (ntl + kNK - 1) / kNK;        // tile steps (the same for both rings)
  const int fr = lane & 15, fq = lane >> 4;
  char* ring = smem + kg * (S * kSlot);

  // ---- Q^T operand pieces and the mask words of this wave's rows
  uint4 qf[4][RTW];
  uint64_t rowmask[RTW];
  int rho[RTW];
#pragma unroll
  for (int t = 0; t < RTW; ++t) {
    rho[t] = 16 * (rr * RTW + t) + fr;
    const bool valid = rho[t] < R;
    const int i = valid ? rho[t] / G : 0;
    const int hh = valid ? rho[t] - i * G : 0;
    const bf16_t* qp = static_cast<const bf16_t*>(a.q) + ((static_cast<size_t>(b) * a.n_q + i) * a.Hq + g * G + hh) * 128 + fq * 8;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
      qf[ks][t] = valid ? *reinterpret_cast<const uint4*>(qp + ks * 32) : make_uint4(0, 0, 0, 0);
    rowmask[t] = !valid ? 0ull : (a.mask ? a.mask[static_cast<size_t>(b) * a.mask_stride + i] : ((2ull << i) - 1ull));
  }

  // ---- page ids of the segment, copied to LDS once: loads from there do not count against
  // the vector-memory counter that paces the tile loads
  const int ps_shift = 31 - __builtin_clz(a.page_size);
  const int pg0 = s0 >> ps_shift;               // first page index of the segment
  if (PAGED) {
    const int npg = ((s1 - 1) >> ps_shift) - pg0 + 1;
    const int32_t* ptab = a.page_table + static_cast<size_t>(b) * a.max_pages + pg0;
    for (int i = threadIdx.x; i < npg; i += 64 * kNK * NR) {
      pg_lds[i] = checked_page(ptab[i], a.n_pages, a.status);   // never leave the pool
    }
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));    // from here on vmcnt counts tile loads only
  __syncthreads();

  // ---- tile loads: the ring's waves take the 16 one-KB pieces of a tile in turn.  Piece j
  // holds keys 4 (j % 8) .. + 3; lane l fetches key 4 (j % 8) + l / 16, 16-byte chunk
  // (l % 16) ^ swizzle(key), and lands at piece base + 16 l, so that LDS entry [key][pos] holds
  // chunk pos ^ swizzle(key).  The lane's byte offset inside a tile does not depend on the tile.
  uint32_t lane_off[(16 + NR - 1) / NR];
#pragma unroll
  for (int u = 0; u < (16 + NR - 1) / NR; ++u) {
    const int key = 4 * ((rr + u * NR) & 7) + fq;
    const int in_row = PAGED ? (key & (a.page_size - 1)) : key;
    const int sw = ((rr + u * NR) & 8) ? swz_v(key) : swz_k(key);   // pieces 8..15 are V
    lane_off[u] = static_cast<uint32_t>(in_row) * 256u + static_cast<uint32_t>((fr ^ sw) << 4);
  }
  const size_t seq_row = PAGED ? 0 : (static_cast<size_t>(b) * a.Hkv + g) * a.l_max;
  auto issue = [&](int it) {
    const int ti = it * kNK + kg;
    if (it >= nit || ti >= ntl) return;        // uniform per wave
    const int t0 = s0 + 32 * ti;
    char* slot = ring + (it % S) * kSlot;
    // rows of the pool that hold the tile's first and second 16 keys (pages of 16 * 2^n
    // tokens: a 32-aligned tile touches at most the page of key 0 and the page of key 16)
    size_t row_a, row_b;
    if (PAGED) {
      const int p1 = min(t0 + 16, s1 - 1);
      const int pg_a = pg_lds[(t0 >> ps_shift) - pg0], pg_b = pg_lds[(p1 >> ps_shift) - pg0];
      row_a = (static_cast<size_t>(pg_a) * a.Hkv + g) * a.page_size;
      row_b = (static_cast<size_t>(pg_b) * a.Hkv + g) * a.page_size;
    } else {
      row_a = row_b = seq_row;
    }
    if (t0 + 32 <= s1) {
      // whole tile inside the range: uniform base per piece + the lane's constant offset
      const size_t in_page = PAGED ? static_cast<size_t>(t0 & (a.page_size - 1)) : static_cast<size_t>(t0);
#pragma unroll
      for (int u = 0; u < (16 + NR - 1) / NR; ++u) {
        const int j = rr + u * NR;             // piece: 0..7 K keys 4j.., 8..15 V keys 4(j-8)..
        if (j < 16) {
          const bool second = PAGED && a.page_size == 16 && (j & 4);   // keys 16..31 sit in the next page
          const char* base = static_cast<const char*>(j < 8 ? a.k : a.v) + ((second ? row_b : row_a) + in_page) * 256;
          load_to_lds16(base, lane_off[u], slot + j * 1024);
        }
      }
      return;
    }
    const int page0 = t0 >> ps_shift;
#pragma unroll
    for (int u = 0; u < (16 + NR - 1) / NR; ++u) {
      const int j = rr + u * NR;
      if (j < 16) {
        const int i = j & 7;
        const int key = 4 * i + fq;
        const int p = min(t0 + key, s1 - 1);   // keys past the range are masked in the softmax
        size_t row;
        if (PAGED) row = ((p >> ps_shift) == page0 ? row_a : row_b) + (p & (a.page_size - 1));
        else row = row_a + p;
        const char* src = static_cast<const char*>(j < 8 ? a.k : a.v) + row * 256 + ((fr ^ (j < 8 ? swz_k(key) : swz_v(key))) << 4);
        load_to_lds16(src, slot + j * 1024);
      }
    }
  };
  constexpr int kPiecesMin = 16 / NR;          // pieces every wave of a ring issues per tile, at least

  f32x4_t oacc[8][RTW];
  float m_run[RTW], l_run[RTW];
#pragma unroll
  for (int t = 0; t < RTW; ++t) {
    m_run[t] = -INFINITY;
    l_run[t] = 0.f;
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) oacc[dt][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  const float sl2 = a.scale * 1.44269504088896340736f;  // scores are kept in log2 units

#pragma unroll
  for (int it = 0; it < S - 1; ++it) issue(it);

  for (int it = 0; it < nit; ++it) {
    // this wave's pieces of tile `it` have landed once at most the pieces of the S-2 tiles
    // issued after it are outstanding (loads return in order); near the end simply wait for all
    if (S > 2 && it + S - 1 < nit) __builtin_amdgcn_s_waitcnt(vmcnt_imm((S - 2) * kPiecesMin));
    else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    // plain barrier (no memory fence: a fence would wait for the loads still in flight); the
    // wave-scope fences only keep the compiler from moving LDS accesses across it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_barrier();              // tile `it` complete; slot of tile it-1 free
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    issue(it + S - 1);
    const int ti = it * kNK + kg;
    if (ti >= ntl) continue;
    const int t0 = s0 + 32 * ti;
    const char* k_lds = ring + (it % S) * kSlot;
    const char* v_lds = k_lds + 8192;

    // ---- S^T = K Q^T for the two 16-key halves.  The K operand reads run kKAhead reads ahead of the
    // matrix instructions that use them, and the first V operand reads are issued here as well (they do
    // not depend on the softmax).  The scheduler is kept from sinking the reads back to their uses: left
    // alone it aims at the fewest registers and leaves one LDS round trip per matrix instruction exposed.
    f32x4_t sacc[2][RTW];
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int t = 0; t < RTW; ++t) sacc[j][t] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    auto kread = [&](int i) {       // read i: k step i / 2, key half i % 2
      const int ks = i >> 1, j = i & 1;
      return reinterpret_cast<const uint4*>(k_lds)[(16 * j + fr) * 16 + ((4 * ks + fq) ^ fr)];
    };
    // Transpose load of V: within 16 lanes, lane i = 4 e + c points at key e's four values
    // d0 + 4c .. d0 + 4c + 3 and lane j receives column d0 + j of keys e = 0..3.  Two loads give the
    // 8 keys of the operand in the order P^T uses: 4q..4q+3 of the first half, then of the second half.
    const int ve = fr >> 2, vc = fr & 3;
    const int key0 = 4 * fq + ve, key1 = 16 + key0;
    s16x4_t vlo[8], vhi[8];
    auto vread = [&](int dt) {
      const int chunk = 2 * dt + (vc >> 1);
      const char* p0 = v_lds + key0 * 256 + ((chunk ^ swz_v(key0)) << 4) + ((vc & 1) << 3);
      const char* p1 = v_lds + key1 * 256 + ((chunk ^ swz_v(key1)) << 4) + ((vc & 1) << 3);
      vlo[dt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(lds_ptr_t)p0);
      vhi[dt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(lds_ptr_t)p1);
    };
    uint4 kf[8];
#pragma unroll
    for (int i = 0; i < kKAhead; ++i) kf[i] = kread(i);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (i + kKAhead < 8) kf[i + kKAhead] = kread(i + kKAhead);
      if (i >= 8 - kVAhead) vread(i - (8 - kVAhead));      // the last K steps also start the V reads
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < RTW; ++t)
        sacc[i & 1][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, kf[i]),
                                                                __builtin_bit_cast(bf16x8_t, qf[i >> 1][t]), sacc[i & 1][t], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }

    // ---- online softmax; lane (row, q) owns keys t0 + 16 j + 4 q + e of its row
    const bool need_mask = t0 + 32 > min(L, s1);
    uint4 pf[RTW];
    float alpha[RTW];
    bool rescale = false;
#pragma unroll
    for (int t = 0; t < RTW; ++t) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) x[4 * j + e] = sacc[j][t][e] * sl2;
      if (need_mask) {
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int p = t0 + 16 * j + 4 * fq + e;
            bool vis = p < s1;
            if (vis && p >= L) vis = (rowmask[t] >> (p - L)) & 1ull;
            if (!vis) x[4 * j + e] = -INFINITY;
          }
      }
      float mt = fmaxf(fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3])), fmaxf(fmaxf(x[4], x[5]), fmaxf(x[6], x[7])));
      mt = quad_row_max(mt);
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
      pf[t] = make_uint4(pack_bf16x2(pr[0], pr[1]), pack_bf16x2(pr[2], pr[3]), pack_bf16x2(pr[4], pr[5]),
                         pack_bf16x2(pr[6], pr[7]));
      l_run[t] = l_run[t] * al + (((pr[0] + pr[1]) + (pr[2] + pr[3])) + ((pr[4] + pr[5]) + (pr[6] + pr[7])));
      m_run[t] = m_new;
      alpha[t] = al;
      rescale = rescale || (al != 1.f);
    }
    if (__builtin_amdgcn_ballot_w64(rescale) != 0ull) {
#pragma unroll
      for (int t = 0; t < RTW; ++t)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          oacc[dt][t][0] *= alpha[t]; oacc[dt][t][1] *= alpha[t];
          oacc[dt][t][2] *= alpha[t]; oacc[dt][t][3] *= alpha[t];
        }
    }

    // ---- O^T += V^T P^T, the V operand reads kVAhead matrix instructions ahead
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) {
      if (dt + kVAhead < 8) vread(dt + kVAhead);
      __builtin_amdgcn_sched_barrier(0);
      const uint2 l2 = __builtin_bit_cast(uint2, vlo[dt]), h2 = __builtin_bit_cast(uint2, vhi[dt]);
      const bf16x8_t va = __builtin_bit_cast(bf16x8_t, make_uint4(l2.x, l2.y, h2.x, h2.y));
#pragma unroll
      for (int t = 0; t < RTW; ++t)
        oacc[dt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, __builtin_bit_cast(bf16x8_t, pf[t]), oacc[dt][t], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));

  // ---- merge the two rings of each row in a fixed order, then one partial per workgroup
  float* o_lds = reinterpret_cast<float*>(smem);   // merge buffer [RP][kORow], overlays the rings
#pragma unroll
  for (int t = 0; t < RTW; ++t) {
    float l = l_run[t];
    l += __shfl_xor(l, 16, 64);
    l += __shfl_xor(l, 32, 64);
    if (fq == 0) {
      ml_lds[(kg * RP + rho[t]) * 2 + 0] = m_run[t];
      ml_lds[(kg * RP + rho[t]) * 2 + 1] = l;
    }
  }
  __syncthreads();   // also: every wave is done with the rings
  const size_t unit = static_cast<size_t>(blockIdx.x) + static_cast<size_t>(b) * a.Hkv + g;   // partial slot of segment (w, u)
  float fself[RTW];
#pragma unroll
  for (int t = 0; t < RTW; ++t) {
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < kNK; ++w) mm = fmaxf(mm, ml_lds[(w * RP + rho[t]) * 2]);
    float lt = 0.f;
    fself[t] = 0.f;
#pragma unroll
    for (int w = 0; w < kNK; ++w) {
      const float mw = ml_lds[(w * RP + rho[t]) * 2];
      const float fw = (mw == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mw - mm);
      lt = fmaf(fw, ml_lds[(w * RP + rho[t]) * 2 + 1], lt);
      if (w == kg) fself[t] = fw;
    }
    if (kg == 0 && fq == 0 && rho[t] < R) {
      a.part_ml[(unit * R + rho[t]) * 2 + 0] = mm;
      a.part_ml[(unit * R + rho[t]) * 2 + 1] = lt;
    }
  }
  for (int w = 0; w < kNK; ++w) {
    if (kg == w) {
#pragma unroll
      for (int t = 0; t < RTW; ++t)
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
          float4* dst = reinterpret_cast<float4*>(o_lds + rho[t] * kORow + 16 * dt + 4 * fq);
          float4 v = make_float4(oacc[dt][t][0] * fself[t], oacc[dt][t][1] * fself[t], oacc[dt][t][2] * fself[t],
                                 oacc[dt][t][3] * fself[t]);
          if (w != 0) {
            const float4 o = *dst;
            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
          }
          *dst = v;
        }
    }
    __syncthreads();
  }
  for (int idx = threadIdx.x; idx < R * 32; idx += 64 * kNK * NR) {
    const int r = idx >> 5, c4 = idx & 31;
    *reinterpret_cast<float4*>(a.part_o + (unit * R + r) * 128 + c4 * 4) =
        *reinterpret_cast<const float4*>(o_lds + r * kORow + c4 * 4);
  }
  // a further segment refills the rings under the merge buffer: its first loads are issued after
  // the barrier that follows the page-id copy, which every thread reaches after these reads
  }
}

template <int NR, int RTW, int S, bool PAGED>
hipError_t launch_one(const AttnArgs& a, hipStream_t s) {
  static_assert(NR * RTW <= 8, "at most 128 query rows");
  // set once per process; a function-local static is initialised under the language's own lock,
  // so first calls from several host threads are safe
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_ring<NR, RTW, S, PAGED>),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((k_attn_ring<NR, RTW, S, PAGED>), dim3(a.wgrid), dim3(64 * kNK * NR), attn_mfma_lds_bytes(a), s, a);
  return hipGetLastError();
}

template <int NR, int RTW>
hipError_t launch_nr(const AttnArgs& a, hipStream_t s) {
  if constexpr (NR >= kBigFrom)
    return a.paged ? launch_one<NR, RTW, kBigStages, true>(a, s) : launch_one<NR, RTW, kBigStages, false>(a, s);
  return a.paged ? launch_one<NR, RTW, 2, true>(a, s) : launch_one<NR, RTW, 2, false>(a, s);
}

}  // namespace

bool attn_mfma_supported(const AttnArgs& a) {
  const int R = (a.Hq / a.Hkv) * a.n_q;
  const bool pow2 = (a.page_size & (a.page_size - 1)) == 0;
  return a.dtype == 1 && a.d == 128 && R <= 128 && (!a.paged || (pow2 && a.page_size >= 16));
}

// Workgroups per compute unit and ring depth (see kBigFrom).
int attn_mfma_per_cu(const AttnArgs& a) { return ((a.Hq / a.Hkv) * a.n_q + 15) / 16 >= kBigFrom ? 1 : 2; }
int attn_mfma_stages(const AttnArgs& a) { return attn_mfma_per_cu(a) == 1 ? kBigStages : 2; }

size_t attn_mfma_lds_bytes(const AttnArgs& a) {
  const int rp = 16 * (((a.Hq / a.Hkv) * a.n_q + 15) / 16);
  return static_cast<size_t>(front_bytes(rp, a.stages)) + static_cast<size_t>(kNK) * rp * 2 * sizeof(float) +
         static_cast<size_t>(sched_words(a.B)) * sizeof(int) + (a.paged ? static_cast<size_t>(kMaxChunkPages + 1) * sizeof(int) : 0);
}

int attn_mfma_max_chunk(const AttnArgs& a) { return a.paged ? kMaxChunkPages * a.page_size : (1 << 30); }

hipError_t launch_attn_mfma(const AttnArgs& a, hipStream_t s) {
  const int R = (a.Hq / a.Hkv) * a.n_q;
  switch ((R + 15) / 16) {
    case 1: return launch_nr<1, 1>(a, s);
    case 2: return launch_nr<2, 1>(a, s);
    case 3: return launch_nr<3, 1>(a, s);
    case 4: return launch_nr<4, 1>(a, s);
    case 5: return launch_nr<5, 1>(a, s);
    case 6: return launch_nr<6, 1>(a, s);
    case 7: return launch_nr<7, 1>(a, s);
    case 8: return launch_nr<8, 1>(a, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sx
