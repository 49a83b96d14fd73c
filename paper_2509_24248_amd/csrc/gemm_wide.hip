// LM-head GEMM + argmax over many activation rows (more than 32: the verification block of a
// batch), bf16 x bf16 -> fp32, logits never stored (Alg. 1, target tokens of the block).
//
// With that many rows the activations no longer fit beside the weights: staging them block by
// block in LDS, as the kernel for fewer rows does, fills the LDS with activations, leaves two
// 4 KB weight blocks per wave in flight and makes every wave read all activations from LDS for
// each 16-row weight tile.  Here the roles are swapped:
//   - one workgroup per compute unit walks an equal share of the weight tiles (16 rows each),
//     whatever the vocabulary size: no rounds of workgroups, no refill of the pipeline between them;
//   - the WEIGHTS pass through an LDS ring of S stages, one 128-k block of TG tiles per stage.  Two
//     producer waves do nothing but bring stages in with direct global->LDS loads (16 bytes per
//     lane, streaming), S-1 stages ahead; their load counters hold nothing else, so three stages
//     stay in flight across the barriers;
//   - the ACTIVATIONS stay in registers: consumer wave c owns RTW 16-row tiles of the rows and
//     loads their operand pieces of the next k block (L2 hits) while it works on this one, from a
//     copy of the activations in operand order (k_pack_act) so that a load covers whole cache lines;
//   - a pass takes 2 TG tiles through all k blocks, the two halves of a k block one after the other,
//     so the activation pieces of a k block are fetched once for 256 weight rows; every consumer
//     multiplies every weight tile of a stage with its own rows: one LDS read (the transposed
//     weight operand) feeds RTW matrix instructions.
// One workgroup barrier per stage hands a landed stage to the consumers and the stage read
// before it back to the producers.  The epilogue of a pass reduces each activation row's logits
// over a half's 16 TG weight rows to one (value, index) candidate.
// What bounds it (measured by leaving parts out, 144 rows, V = 151936, D = 5120, event times of a
// stand-alone loop): the producers alone stream at 7 TB/s (230 us), the consumers alone (no weight
// stream) take 225 us, together 340 us whether the ring has three, four or five stages; of that the
// LDS reads and barriers cost 45 us, the matrix instructions 45 us, the activation loads 25 us
// (80 us before they covered whole cache lines: a wave's load straight from the row-major matrix is
// 16 rows x 64 bytes, and such half-line requests, not their bytes, were the cost).  One row of
// workgroups per 128 weight rows, refilled five times per compute unit, took 437 us in the same loop.
// At 56 and 64 rows (V = 151936, D = 4096) it takes 241 us where the LDS-staged kernel took 272 us; up to
// 32 rows (one consumer wave) the LDS-staged kernel is as fast or faster (8 / 16 / 32 rows, D = 5120: 236 /
// 242 / 271 us against 247 / 249 / 272 us), so this kernel starts at 33 rows.
#include "common.hpp"
#include "kernels.hpp"

#include <limits.h>

#include <algorithm>

namespace sx {

namespace {

constexpr int kProducers = 2;

typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | (((n >> 4) & 3) << 14); }

// Direct global -> LDS load, 16 bytes per lane: lane l's bytes land at lds_base + 16 l (lds_base
// wave-uniform).  Written as an instruction so that the kernel paces these loads itself with
// s_waitcnt vmcnt and a barrier.  "nt": the weights are read once.
__device__ __forceinline__ void load_to_lds16(const void* src, const void* lds_base) {
  const uint32_t l = static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_ptr_t)lds_base));
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off nt" ::"s"(l), "v"(src) : "memory");
}

// The stages of a workgroup in the order they pass through the ring.  The workgroup's tiles
// [t_lo, t_hi) are cut into "halves" of TG tiles; a pass takes two halves (the last pass one, if the
// count is odd) through all k blocks, the halves of a k block one after the other, so that the
// consumers fetch their activation pieces of a k block once for 2 TG tiles.
struct StageCursor {
  int half0, nh, kb, h;   // first half and number of halves of the current pass; k block; half within the pass
  static constexpr int kNH = 2;
  __device__ __forceinline__ void start(int nhalf) { half0 = 0; nh = min(kNH, nhalf); kb = 0; h = 0; }
  __device__ __forceinline__ void advance(int nhalf, int KB) {
    if (++h < nh) return;
    h = 0;
    if (++kb < KB) return;
    kb = 0;
    half0 += nh;
    nh = min(kNH, nhalf - half0);
  }
};

// The consumer side of k_head_wide for a wave that owns RT row tiles (from row tile rt0 on) and, of
// every half, the JN weight tiles from jc0 on (all TG, or half of them when a last odd row tile is
// shared by two waves): one barrier per stage, an argmax epilogue per pass.  A row has two candidate
// slots per half, one per column half; a wave that covers the whole half fills the second with nothing.
template <int RT, int JN, int TG, int S>
struct Consumer {
  static constexpr int kStage = TG * 4096;
  const GemmArgs& g;
  char* lds;
  int rt0, jc0, fr, fq, t_lo, t_hi, KB, slots;
  const uint4* apack[RT];   // this lane's piece of row tile t in the packed activations, k block 0, k step 0
  size_t kb_stride;         // uint4 entries from one k block to the next
  uint4 bn[RT][2];  // pieces 0 and 1 of the next k block, on their way
  uint4 b[RT][4];   // activation operand pieces of the current k block: row 16 (wv RTW + t) + fr, k = 32 s + 8 fq .. + 7
  int stage_no;     // stages consumed so far: stage i lives in ring slot i % S

  __device__ __forceinline__ Consumer(const GemmArgs& g_, char* lds_, int rt0_, int jc0_, int NT, int lane, int t_lo_, int t_hi_, int KB_, int slots_)
      : g(g_), lds(lds_), rt0(rt0_), jc0(jc0_), fr(lane & 15), fq(lane >> 4), t_lo(t_lo_), t_hi(t_hi_), KB(KB_), slots(slots_), stage_no(0) {
    // packed activations: [k block][row tile][k step][lane] 16-byte pieces (NT row tiles), so that one
    // load instruction of a wave reads 1 KB of consecutive bytes
    kb_stride = static_cast<size_t>(NT) * 256;
#pragma unroll
    for (int t = 0; t < RT; ++t) apack[t] = static_cast<const uint4*>(g.a_packed) + static_cast<size_t>(rt0 + t) * 256 + lane;
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int s = 0; s < 4; ++s) b[t][s] = apack[t][s * 64];
  }

  // one pass: NH halves starting at half `half0`
  template <int NH>
  __device__ __forceinline__ void pass(int half0) {
    f32x4_t acc[RT][NH * JN];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int j = 0; j < NH * JN; ++j) acc[t][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // The waves go through a stage's four k steps in read groups of CH tiles, the operand reads one
    // group ahead of the matrix instructions (k steps outermost: between two matrix instructions on the
    // same accumulator lie those of all other tiles; the scheduler is kept from sinking the reads back
    // to their uses).  The barrier that hands over the next stage sits before the last group's matrix
    // instructions, whose operands are in registers by then: the first reads of the next stage are in
    // flight while those instructions run, so neither the LDS nor the matrix cores idle around a barrier.
    constexpr int CH = 4;                 // tiles per read group
    constexpr int GPS = JN / CH;          // read groups per k step
    constexpr int NCH = 4 * GPS;          // read groups per stage: group c = k step c / GPS, this wave's tiles CH (c % GPS) ..
    uint4 wf[2][CH];
    auto wait_stage = [&]() -> const uint4* {
      __builtin_amdgcn_s_waitcnt(0xC07F);            // lgkmcnt(0): this wave is done reading the stage it leaves
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_s_barrier();                  // the next stage has landed; the one just read is free
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      const uint4* stage = reinterpret_cast<const uint4*>(lds + (stage_no % S) * kStage) + fr * 16;
      ++stage_no;
      return stage;
    };
    auto read_group = [&](uint4 (&dst)[CH], const uint4* stage, int c) {
      const int s = c / GPS, j0 = CH * (c % GPS);
#pragma unroll
      for (int jj = 0; jj < CH; ++jj) dst[jj] = stage[(jc0 + j0 + jj) * 256 + ((4 * s + fq) ^ fr)];
    };
    const uint4* stage = wait_stage();
    read_group(wf[0], stage, 0);
#pragma unroll 1
    for (int kb = 0; kb < KB; ++kb) {
      // the pieces of the next k block (of the first one again after the last: the next pass starts there)
      const size_t noff = static_cast<size_t>(kb + 1 == KB ? 0 : kb + 1) * kb_stride;
#pragma unroll
      for (int h = 0; h < NH; ++h) {
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
          const int s = c / GPS, j0 = CH * (c % GPS);
          if (c + 1 < NCH) {
            read_group(wf[(c + 1) & 1], stage, c + 1);
          } else if (h < NH - 1 || kb + 1 < KB) {
            stage = wait_stage();
            read_group(wf[0], stage, 0);
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int jj = 0; jj < CH; ++jj)
#pragma unroll
            for (int t = 0; t < RT; ++t)
              acc[t][h * JN + j0 + jj] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[c & 1][jj]),
                                                                                 __builtin_bit_cast(bf16x8_t, b[t][s]), acc[t][h * JN + j0 + jj], 0, 0, 0);
          // The next k block's activation pieces (1 KB of consecutive bytes per instruction, L2 hits that
          // take more than a microsecond under the weight stream).  Pieces 0 and 1, which the next block
          // needs first, are requested into spare registers at the start of this block and moved over when
          // the last half is done with the old ones; pieces 2 and 3 are requested into their own place as
          // soon as the last half is done with them.
          if (h == 0 && c == 0) {
#pragma unroll
            for (int t = 0; t < RT; ++t) {
              bn[t][0] = apack[t][noff];
              bn[t][1] = apack[t][noff + 64];
            }
          }
          if (h == NH - 1 && (c + 1) % GPS == 0) {
#pragma unroll
            for (int t = 0; t < RT; ++t) {
              if (s < 2) b[t][s] = bn[t][s];
              else b[t][s] = apack[t][noff + s * 64];
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
    }

    // ---- epilogue: lane (c = lane % 16, q = lane / 16) holds weight rows 16 (tile0 + j) + 4 q + i of
    // activation row 16 (rt0 + t) + c; rows below V enter the argmax (lowest index on ties), the
    // rows V.. are the widened head's extra rows.  One candidate per row, half and column half.
    const size_t nslot = static_cast<size_t>(gridDim.x) * slots * 2;
#pragma unroll
    for (int h = 0; h < NH; ++h) {
      const int tile0 = t_lo + (half0 + h) * TG + jc0;      // this wave's first tile of the half
#pragma unroll
      for (int t = 0; t < RT; ++t) {
        const int m = 16 * (rt0 + t) + fr;
        const bool owner = m < g.M;
        float bv = -INFINITY;
        int bi = INT_MAX;
        // tiles that lie wholly inside the share and below the signal rows (all but the last of a
        // launch) need no checks per element: the consumers stand still during the epilogue while
        // the ring fills up, so its length counts
        const bool plain = !g.logits_dbg && tile0 + JN <= t_hi && (tile0 + JN) * 16 <= g.V;    // uniform
        if (plain) {
          const int nb = tile0 * 16 + 4 * fq;
#pragma unroll
          for (int j = 0; j < JN; ++j) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float val = acc[t][h * JN + j][i];
              const bool up = val > bv;                      // n grows with j and i: '>' keeps the lowest index
              bv = up ? val : bv;
              bi = up ? nb + 16 * j + i : bi;
            }
          }
        } else {
#pragma unroll
          for (int j = 0; j < JN; ++j) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const int n = (tile0 + j) * 16 + 4 * fq + i;
              const float val = acc[t][h * JN + j][i];
              if (owner && tile0 + j < t_hi && n < g.N) {    // (tiles past the workgroup's range hold a copy of its last tile)
                if (n < g.V) {
                  if (g.logits_dbg) g.logits_dbg[static_cast<size_t>(m) * g.V + n] = val;
                  if (val > bv) { bv = val; bi = n; }
                } else if (g.extra_out) {
                  g.extra_out[m * g.n_extra + (n - g.V)] = val;
                }
              }
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
          const size_t at = static_cast<size_t>(m) * nslot + (static_cast<size_t>(blockIdx.x) * slots + (half0 + h)) * 2;
          g.part_val[at + (jc0 ? 1 : 0)] = bv;
          g.part_idx[at + (jc0 ? 1 : 0)] = bi;
          if (JN == TG) {
            g.part_val[at + 1] = -INFINITY;
            g.part_idx[at + 1] = INT_MAX;
          }
        }
      }
    }
  }

  __device__ __forceinline__ void run() {
    const int nhalf = (t_hi - t_lo + TG - 1) / TG;
#pragma unroll 1
    for (int half0 = 0; half0 < nhalf; half0 += 2) {
      if (half0 + 1 < nhalf) pass<2>(half0);
      else pass<1>(half0);
    }
    // candidate slots this workgroup does not use (its share of the tiles is one half shorter than the longest)
    if (fq == 0 && jc0 == 0) {
      const size_t nslot = static_cast<size_t>(gridDim.x) * slots * 2;
      for (int q = nhalf; q < slots; ++q)
#pragma unroll
        for (int t = 0; t < RT; ++t) {
          const int m = 16 * (rt0 + t) + fr;
          if (m < g.M) {
            const size_t at = static_cast<size_t>(m) * nslot + (static_cast<size_t>(blockIdx.x) * slots + q) * 2;
            g.part_val[at] = g.part_val[at + 1] = -INFINITY;
            g.part_idx[at] = g.part_idx[at + 1] = INT_MAX;
          }
        }
    }
  }
};

// Activations [M, K] bf16 -> operand pieces [k block][row tile][k step][lane]: lane (c = lane % 16,
// q = lane / 16) of piece (kb, tile, s) holds row 16 tile + c, k = 128 kb + 32 s + 8 q .. + 7; rows
// from M on are zero.  The consumers of k_head_wide then fetch a k block's pieces with loads that
// cover whole cache lines: read straight from the row-major matrix, the same pieces are 16 rows x
// 64 bytes per instruction, and those half-line requests, not their bytes, were what the
// activations cost (144 rows: 80 us of 395 with them, 29 us with full-line loads of the same bytes).
__global__ __launch_bounds__(256) void k_pack_act(const bf16_t* __restrict__ src, uint4* __restrict__ dst, int M, int K, int NT) {
  const int lane = threadIdx.x & 63;
  const int unit = blockIdx.x * 4 + (threadIdx.x >> 6);     // (kb, tile)
  const int KB = K >> 7;
  if (unit >= KB * NT) return;
  const int kb = unit / NT, tile = unit - kb * NT;
  const int m = 16 * tile + (lane & 15);
  const bf16_t* row = src + static_cast<size_t>(m < M ? m : 0) * K + 128 * kb + 8 * (lane >> 4);
  uint4 v[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) v[s] = *reinterpret_cast<const uint4*>(row + 32 * s);
#pragma unroll
  for (int s = 0; s < 4; ++s) dst[(static_cast<size_t>(unit) * 4 + s) * 64 + lane] = m < M ? v[s] : uint4{0u, 0u, 0u, 0u};
}

// NC consumer waves of RTW row tiles, then the producers; SPLIT: the last consumer's second row tile does not
// exist (an odd number of row tiles), and its one tile is shared with a further wave after the producers,
// each taking half of the columns: no SIMD then carries three row tiles' worth of matrix instructions.
template <int NC, int RTW, int TG, int S, bool SPLIT>
__global__ __launch_bounds__(64 * (NC + kProducers + (SPLIT ? 1 : 0))) void k_head_wide(const GemmArgs g) {
  static_assert((4 * TG) % kProducers == 0, "the pieces of a stage are dealt evenly to the producers");
  constexpr int PP = 4 * TG / kProducers;       // 1 KB pieces (4 weight rows x 256 bytes) per producer and stage
  static_assert((S - 2) * PP < 64, "the load counter has six bits");
  constexpr int kStage = TG * 4096;             // bytes of a stage: TG tiles of 16 rows x 128 k
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ntiles = (g.N + 15) >> 4;
  // this workgroup's share of the weight tiles: equal shares whatever the vocabulary size
  const int t_lo = static_cast<int>(static_cast<int64_t>(blockIdx.x) * ntiles / gridDim.x);
  const int t_hi = static_cast<int>(static_cast<int64_t>(blockIdx.x + 1) * ntiles / gridDim.x);
  const int nhalf = (t_hi - t_lo + TG - 1) / TG;
  const int KB = g.K >> 7;
  const int total = nhalf * KB;                 // stages of this workgroup
  const size_t row_bytes = static_cast<size_t>(g.K) * 2;

  if (wv >= NC && wv < NC + kProducers) {
    // ------------------------------------------------------------------ producer
    // piece j of a stage = rows 4 (j % 4) .. + 3 of tile j / 4; lane l fetches row 4 (j % 4) + l / 16,
    // 16-byte piece (l % 16) ^ row and lands at piece base + 16 l, so that tile entry [row][pos]
    // holds piece pos ^ row: the consumers' per-row operand reads then touch 16 distinct slots.
    // Every stage is TG tiles: past the workgroup's last tile that tile is fetched again (an L2 hit),
    // so that every stage counts the same number of loads; the consumers mask those copies.
    const int pw = wv - NC;
    StageCursor cur;
    cur.start(nhalf);
    auto issue = [&](int slot) {
      char* stage = lds + slot * kStage;
      const int tile0 = t_lo + (cur.half0 + cur.h) * TG;
#pragma unroll
      for (int u = 0; u < PP; ++u) {
        const int j = pw + u * kProducers;
        const int r = 4 * (j & 3) + (lane >> 4);
        const int tile = min(tile0 + (j >> 2), t_hi - 1);
        const int row = min(tile * 16 + r, g.N - 1);               // rows past the end repeat the last one, masked later
        const char* src = static_cast<const char*>(g.w[0]) + static_cast<size_t>(row) * row_bytes + (((lane & 15) ^ r) << 4) +
                          (static_cast<size_t>(cur.kb) << 8);
        load_to_lds16(src, stage + j * 1024);
      }
      cur.advance(nhalf, KB);
    };
    int issued = 0;
    for (; issued < S - 1 && issued < total; ++issued) issue(issued % S);
    for (int i = 0; i < total; ++i) {
      // this wave's pieces of stage i have landed once at most the pieces of the S-2 stages issued
      // after it are outstanding (loads return in order); near the end simply wait for all
      if (i + S - 1 < total) __builtin_amdgcn_s_waitcnt(vmcnt_imm((S - 2) * PP));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_s_barrier();              // stage i is complete; the slot of stage i-1 is free
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      if (issued < total) {
        issue(issued % S);
        ++issued;
      }
    }
    return;
  }

  // -------------------------------------------------------------------- consumer
  constexpr int NT = NC * RTW;     // row tiles of the packed activations
  if constexpr (SPLIT) {
    static_assert(RTW == 2, "a split last tile is the first of a pair");
    if (wv == NC - 1) Consumer<1, TG / 2, TG, S>(g, lds, (NC - 1) * RTW, 0, NT, lane, t_lo, t_hi, KB, g.wide_slots).run();
    else if (wv > NC) Consumer<1, TG / 2, TG, S>(g, lds, (NC - 1) * RTW, TG / 2, NT, lane, t_lo, t_hi, KB, g.wide_slots).run();
    else Consumer<RTW, TG, TG, S>(g, lds, wv * RTW, 0, NT, lane, t_lo, t_hi, KB, g.wide_slots).run();
  } else {
    Consumer<RTW, TG, TG, S>(g, lds, wv * RTW, 0, NT, lane, t_lo, t_hi, KB, g.wide_slots).run();
  }
}

// Eight tiles (128 weight rows, 32 KB) per stage and four stages: 96 KB in flight per compute unit.
// Measured at 144 rows, V = 151936, D = 5120: three and five stages the same; three consumer waves of
// three row tiles with one half per pass no faster (fewer LDS reads, more activation loads); the ninth
// row tile shared by two waves instead of one wave next to a full consumer on its SIMD: 1.5 % faster.
constexpr int kWideTiles = 8, kWideStages = 4;

template <int NC, int RTW, bool SPLIT>
hipError_t launch_wide_as(const GemmArgs& g, hipStream_t s) {
  constexpr int TG = kWideTiles, S = kWideStages;
  // set once per process; a function-local static is initialised under the language's own lock
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_head_wide<NC, RTW, TG, S, SPLIT>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr != hipSuccess) return attr;
  const int units = (g.K >> 7) * NC * RTW;
  hipLaunchKernelGGL(k_pack_act, dim3((units + 3) / 4), dim3(256), 0, s, static_cast<const bf16_t*>(g.a_src),
                     static_cast<uint4*>(g.a_packed), g.M, g.K, NC * RTW);
  hipLaunchKernelGGL((k_head_wide<NC, RTW, TG, S, SPLIT>), dim3(g.wide_w), dim3(64 * (NC + kProducers + (SPLIT ? 1 : 0))),
                     static_cast<size_t>(S) * TG * 4096, s, g);
  return hipGetLastError();
}

// an odd number of 16-row tiles: the last one is shared by two waves
template <int NC, int RTW>
hipError_t launch_wide(const GemmArgs& g, hipStream_t s) {
  return ((g.M + 15) / 16) % 2 ? launch_wide_as<NC, RTW, true>(g, s) : launch_wide_as<NC, RTW, false>(g, s);
}

}  // namespace

bool head_wide_supported(const GemmArgs& g) {
  return g.V >= 0 && g.planes == 1 && g.top_b <= 1 && g.M > 32 && g.M <= 160 && g.K % 128 == 0 && g.nseg == 1;
}

// One workgroup per compute unit, each walking an equal share of the weight tiles (at least one
// stage's worth); candidate slots per workgroup = the halves of the longest share.
void head_wide_plan(GemmArgs& g, int num_cus) {
  g.wide = head_wide_supported(g) ? 1 : 0;
  if (!g.wide) return;
  const int ntiles = gemm_ntiles(g.N);
  g.wide_w = std::max(1, std::min(num_cus, ntiles / kWideTiles));
  g.wide_slots = ((ntiles + g.wide_w - 1) / g.wide_w + kWideTiles - 1) / kWideTiles;
}

int head_wide_groups(const GemmArgs& g) { return g.wide_w * g.wide_slots * 2; }

// bytes of the packed activations: the row tiles the consumer waves cover (32 rows each) x K
size_t head_wide_pack_bytes(const GemmArgs& g) { return g.wide ? static_cast<size_t>((g.M + 31) / 32) * 32 * g.K * 2 : 0; }

hipError_t launch_head_wide(const GemmArgs& g, hipStream_t s) {
  if (!head_wide_supported(g) || g.a_mode != 1 || g.wide_w < 1 || !g.a_packed) return hipErrorInvalidValue;
  switch ((g.M + 31) / 32) {
    case 2: return launch_wide<2, 2>(g, s);      // 33 ..  64 rows
    case 3: return launch_wide<3, 2>(g, s);      // 65 ..  96
    case 4: return launch_wide<4, 2>(g, s);      // 97 .. 128
    case 5: return launch_wide<5, 2>(g, s);      // 129 .. 160
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sx
