// LM-head GEMM + argmax over many activation rows (more than 64: the verification block of a
// large batch), bf16 x bf16 -> fp32, logits never stored (Alg. 1, target tokens of the block).
//
// With that many rows the activations no longer fit beside the weights: staging them block by
// block in LDS, as the kernel for fewer rows does, fills the LDS with activations, leaves two
// 4 KB weight blocks per wave in flight and makes every wave read all activations from LDS for
// each 16-row weight tile.  Here the roles are swapped:
//   - the WEIGHTS of the workgroup's TG tiles (16 rows each) pass through an LDS ring of S stages,
//     one 128-k block of all TG tiles per stage.  Two producer waves do nothing but bring stages
//     in with direct global->LDS loads (16 bytes per lane, streaming), S-1 stages ahead; their
//     load counters hold nothing else, so three stages stay in flight across the barriers.
//   - the ACTIVATIONS stay in registers: consumer wave c owns RTW 16-row tiles of the rows and
//     loads their operand pieces of the next k block (L2 hits) while it works on this one.
//   - every consumer multiplies every weight tile of the stage with its own rows: one LDS read
//     (the transposed weight operand) feeds RTW matrix instructions.
// One workgroup barrier per k block hands a landed stage to the consumers and the stage consumed
// one block earlier back to the producers.
// What bounds it (measured by leaving parts out, 144 rows): the weight stream alone runs at
// 5.8 TB/s; the matrix instructions and the LDS reads cost little once the reads are issued a
// k step ahead; the rest is the activations, which every workgroup fetches again from L2 for every
// k block (40 KB per 32 KB of weights: halving them took 438 -> 365 us, a quarter 320 us).  The epilogue reduces each activation row's logits
// over the workgroup's 16 TG weight rows to one (value, index) candidate.
#include "common.hpp"
#include "kernels.hpp"

#include <limits.h>

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

// The consumer side of k_head_wide for a wave that owns RT row tiles (its rows start at
// 16 * wv * RTW): KB steps, one barrier each, then the argmax epilogue.
template <int RT, int RTW, int TG, int S>
__device__ __forceinline__ void consume(const GemmArgs& g, char* lds, int wv, int lane, int tile0, int ntiles, int KB) {
  constexpr int kStage = TG * 4096;
  const int fr = lane & 15, fq = lane >> 4;
  // activation operand pieces of one 128-k block: row 16 (wv RTW + t) + fr, k = 32 s + 8 fq .. + 7
  // (a row past the last one reads row 0 instead: its accumulator column is that lane's own and is
  // never written out, and selecting zeros here would make the wave wait for the loads it has only
  // just issued)
  const bf16_t* arow[RT];
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int m = 16 * (wv * RTW + t) + fr;
    arow[t] = static_cast<const bf16_t*>(g.a_src) + static_cast<size_t>(m < g.M ? m : 0) * g.K + 8 * fq;
  }
  uint4 bA[RT][4], bB[RT][4];
  auto fetch = [&](uint4 (&dst)[RT][4], int kb) {
    const size_t off = static_cast<size_t>(min(kb, KB - 1)) << 7;     // past the end: the last block again, unused
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
      for (int s = 0; s < 4; ++s) dst[t][s] = *reinterpret_cast<const uint4*>(arow[t] + off + 32 * s);
  };
  f32x4_t acc[RT][TG];
#pragma unroll
  for (int t = 0; t < RT; ++t)
#pragma unroll
    for (int j = 0; j < TG; ++j) acc[t][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  auto step = [&](uint4 (&cur)[RT][4], uint4 (&nxt)[RT][4], int kb) {
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));    // this wave's loads are activation pieces only: block kb is here
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_s_barrier();                // stage kb has landed
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    fetch(nxt, kb + 1);
    const uint4* stage = reinterpret_cast<const uint4*>(lds + (kb % S) * kStage) + fr * 16;
    // k steps outermost: between two matrix instructions on the same accumulator lie those of all
    // other tiles (an accumulator used again right away stalls for the instruction's full latency).
    // The TG operand reads of the next k step are issued before this k step's matrix instructions,
    // and the scheduler is kept from sinking them back to their uses (left alone it keeps one read
    // ahead of each matrix instruction, which exposes the LDS latency TG * 4 times per block).
    uint4 wf[2][TG];
#pragma unroll
    for (int j = 0; j < TG; ++j) wf[0][j] = stage[j * 256 + (fq ^ fr)];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      if (s < 3) {
#pragma unroll
        for (int j = 0; j < TG; ++j) wf[(s + 1) & 1][j] = stage[j * 256 + ((4 * (s + 1) + fq) ^ fr)];
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < TG; ++j)
#pragma unroll
        for (int t = 0; t < RT; ++t)
          acc[t][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, wf[s & 1][j]), __builtin_bit_cast(bf16x8_t, cur[t][s]),
                                                              acc[t][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // (an odd block count would need a half step: the launcher takes even counts only)
  fetch(bA, 0);
  for (int kb = 0; kb < KB; kb += 2) {
    step(bA, bB, kb);
    step(bB, bA, kb + 1);
  }

  // ---- epilogue: lane (c = lane % 16, q = lane / 16) holds weight rows 16 (tile0 + j) + 4 q + i of
  // activation row 16 (wv RTW + t) + c; rows below V enter the argmax (lowest index on ties), the
  // rows V.. are the widened head's extra rows
#pragma unroll
  for (int t = 0; t < RT; ++t) {
    const int m = 16 * (wv * RTW + t) + fr;
    const bool owner = m < g.M;
    float bv = -INFINITY;
    int bi = INT_MAX;
#pragma unroll
    for (int j = 0; j < TG; ++j) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = (tile0 + j) * 16 + 4 * fq + i;
        const float val = acc[t][j][i];
        if (owner && tile0 + j < ntiles && n < g.N) {
          if (n < g.V) {
            if (g.logits_dbg) g.logits_dbg[static_cast<size_t>(m) * g.V + n] = val;
            if (val > bv) { bv = val; bi = n; }          // n grows with j and i: '>' keeps the lowest index
          } else if (g.extra_out) {
            g.extra_out[m * g.n_extra + (n - g.V)] = val;
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
      g.part_val[static_cast<size_t>(m) * gridDim.x + blockIdx.x] = bv;
      g.part_idx[static_cast<size_t>(m) * gridDim.x + blockIdx.x] = bi;
    }
  }
}

template <int NC, int RTW, int TG, int S>
__global__ __launch_bounds__(64 * (NC + kProducers)) void k_head_wide(const GemmArgs g) {
  static_assert((4 * TG) % kProducers == 0, "the pieces of a stage are dealt evenly to the producers");
  constexpr int PP = 4 * TG / kProducers;       // 1 KB pieces (4 weight rows x 256 bytes) per producer and stage
  static_assert((S - 2) * PP < 64, "the load counter has six bits");
  constexpr int kStage = TG * 4096;             // bytes of a stage: TG tiles of 16 rows x 128 k
  extern __shared__ uint4 lds4[];
  char* lds = reinterpret_cast<char*>(lds4);
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int ntiles = (g.N + 15) >> 4;
  const int tile0 = blockIdx.x * TG;
  const int KB = g.K >> 7;
  const size_t row_bytes = static_cast<size_t>(g.K) * 2;

  if (wv >= NC) {
    // ------------------------------------------------------------------ producer
    // piece j of a stage = rows 4 (j % 4) .. + 3 of tile j / 4; lane l fetches row 4 (j % 4) + l / 16,
    // 16-byte piece (l % 16) ^ row and lands at piece base + 16 l, so that tile entry [row][pos]
    // holds piece pos ^ row: the consumers' per-row operand reads then touch 16 distinct slots
    const int pw = wv - NC;
    const char* src[PP];
#pragma unroll
    for (int u = 0; u < PP; ++u) {
      const int j = pw + u * kProducers;
      const int r = 4 * (j & 3) + (lane >> 4);
      const int row = min((tile0 + (j >> 2)) * 16 + r, g.N - 1);    // rows past the end repeat the last one, masked later
      src[u] = static_cast<const char*>(g.w[0]) + static_cast<size_t>(row) * row_bytes + (((lane & 15) ^ r) << 4);
    }
    auto issue = [&](int kb) {
      if (kb >= KB) return;                      // uniform per wave
      char* stage = lds + (kb % S) * kStage;
#pragma unroll
      for (int u = 0; u < PP; ++u) load_to_lds16(src[u] + (static_cast<size_t>(kb) << 8), stage + (pw + u * kProducers) * 1024);
    };
#pragma unroll
    for (int kb = 0; kb < S - 1; ++kb) issue(kb);
    for (int kb = 0; kb < KB; ++kb) {
      // this wave's pieces of stage kb have landed once at most the pieces of the S-2 stages issued
      // after it are outstanding (loads return in order); near the end simply wait for all
      if (kb + S - 1 < KB) __builtin_amdgcn_s_waitcnt(vmcnt_imm((S - 2) * PP));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_s_barrier();              // stage kb is complete; the slot of stage kb-1 is free
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
      issue(kb + S - 1);
    }
    return;
  }

  // -------------------------------------------------------------------- consumer
  // a wave whose second row tile lies wholly past the last row works on one tile only
  if (RTW == 2 && 16 * (wv * RTW + 1) >= g.M) consume<1, RTW, TG, S>(g, lds, wv, lane, tile0, ntiles, KB);
  else consume<RTW, RTW, TG, S>(g, lds, wv, lane, tile0, ntiles, KB);
}

// Eight tiles (128 weight rows, 32 KB per stage) and four stages: 96 KB in flight per compute unit.
// Measured at 144 rows, V = 151936, D = 5120: three stages the same, four tiles per stage (two
// workgroups per compute unit) 35 % slower, one row tile per consumer wave (nine consumers) the same.
constexpr int kWideTiles = 8, kWideStages = 4;

template <int NC, int RTW>
hipError_t launch_wide(const GemmArgs& g, hipStream_t s) {
  constexpr int TG = kWideTiles, S = kWideStages;
  // set once per process; a function-local static is initialised under the language's own lock
  static const hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_head_wide<NC, RTW, TG, S>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  if (attr != hipSuccess) return attr;
  hipLaunchKernelGGL((k_head_wide<NC, RTW, TG, S>), dim3(head_wide_groups(g)), dim3(64 * (NC + kProducers)),
                     static_cast<size_t>(S) * TG * 4096, s, g);
  return hipGetLastError();
}

}  // namespace

bool head_wide_supported(const GemmArgs& g) {
  return g.V >= 0 && g.planes == 1 && g.top_b <= 1 && g.M > 64 && g.M <= 160 && g.K % 256 == 0 && g.nseg == 1;
}

int head_wide_groups(const GemmArgs& g) { return (gemm_ntiles(g.N) + kWideTiles - 1) / kWideTiles; }

hipError_t launch_head_wide(const GemmArgs& g, hipStream_t s) {
  if (!head_wide_supported(g) || g.a_mode != 1) return hipErrorInvalidValue;
  switch ((g.M + 31) / 32) {
    case 3: return launch_wide<3, 2>(g, s);      // 65 ..  96 rows
    case 4: return launch_wide<4, 2>(g, s);      // 97 .. 128
    case 5: return launch_wide<5, 2>(g, s);      // 129 .. 160
    default: return hipErrorInvalidValue;
  }
}

}  // namespace sx
