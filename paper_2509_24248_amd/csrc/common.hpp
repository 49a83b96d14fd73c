// Shared device helpers for the SpecExit kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sx {

typedef uint16_t bf16_t;  // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// round to nearest even; inputs here are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

// two floats -> packed bf16 pair (a in the low half), round to nearest even in hardware
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPer16B = 4;
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static constexpr int kPer16B = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// 16-byte vector of storage elements -> floats
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[8]) {
  f[0] = __uint_as_float(v.x << 16); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
  f[2] = __uint_as_float(v.y << 16); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
  f[4] = __uint_as_float(v.z << 16); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
  f[6] = __uint_as_float(v.w << 16); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Maximum over the four lanes l, l ^ 16, l ^ 32, l ^ 48 (the four k groups of a matrix-core
// accumulator column) without an LDS round trip: the swap instructions hand every lane both halves
// of the exchange with its partner row (with both operands equal, the first result holds rows
// 0, 0, 2, 2 and the second rows 1, 1, 3, 3 of 16 lanes; the 32-lane form likewise).
__device__ __forceinline__ float quad_row_max(float v) {
  const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
  const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

// (value, index) pair ordered by larger value, then lower index
__device__ __forceinline__ bool better(float v, int i, float bv, int bi) {
  return v > bv || (v == bv && i < bi);
}

// Data handed from one workgroup to another inside a kernel (split-K partial sums that the
// last workgroup to arrive adds up) is written and read at agent scope: the sc1 forms of the
// store and load go through to the level all compute units of the device share, so no cache
// has to be written back or invalidated as a whole (an agent-scope fence would do both).
// The writer waits for its stores (s_waitcnt vmcnt(0)) before it signals through an atomic.
typedef float f32x4v_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_agent16(float* p, float a, float b, float c, float d) {
  const f32x4v_t v = {a, b, c, d};
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// four independent 16-byte agent-scope loads, waited for together
__device__ __forceinline__ void load_agent16x4(const float* p0, const float* p1, const float* p2, const float* p3,
                                               float4 (&out)[4]) {
  f32x4v_t a, b, c, d;
  asm volatile(
      "global_load_dwordx4 %0, %4, off sc1\n\t"
      "global_load_dwordx4 %1, %5, off sc1\n\t"
      "global_load_dwordx4 %2, %6, off sc1\n\t"
      "global_load_dwordx4 %3, %7, off sc1\n\t"
      "s_waitcnt vmcnt(0)"
      : "=&v"(a), "=&v"(b), "=&v"(c), "=&v"(d)
      : "v"(p0), "v"(p1), "v"(p2), "v"(p3)
      : "memory");
  out[0] = make_float4(a.x, a.y, a.z, a.w);
  out[1] = make_float4(b.x, b.y, b.z, b.w);
  out[2] = make_float4(c.x, c.y, c.z, c.w);
  out[3] = make_float4(d.x, d.y, d.z, d.w);
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

// Values read from device arrays never reach an address unchecked: they are forced into range
// (a bad value then gives a wrong result for its row, never a fault), and the first one seen is
// reported in the caller's device status word when one was given.
constexpr int kStatusBadLength = 1;  // ctx_len / pos < 0 or beyond the cache capacity
constexpr int kStatusBadPage = 2;    // page id outside 0 .. n_pages-1
constexpr int kStatusBadToken = 3;   // token id outside 0 .. V-1
constexpr int kStatusBadNode = 4;    // node id, path entry or row index outside its block

__device__ __forceinline__ void report_status(int* status, int code) {
  if (status) atomicCAS(status, 0, code);
}

__device__ __forceinline__ int checked_page(int page, int64_t n_pages, int* status) {
  if (static_cast<uint32_t>(page) < static_cast<uint32_t>(n_pages)) return page;
  report_status(status, kStatusBadPage);
  return 0;
}

// for writes: a cache entry whose page id is out of range is not written at all
__device__ __forceinline__ bool page_in_pool(int page, int64_t n_pages, int* status) {
  if (static_cast<uint32_t>(page) < static_cast<uint32_t>(n_pages)) return true;
  report_status(status, kStatusBadPage);
  return false;
}

__device__ __forceinline__ int checked_token(int tok, int vocab, int* status) {
  if (static_cast<uint32_t>(tok) < static_cast<uint32_t>(vocab)) return tok;
  report_status(status, kStatusBadToken);
  return 0;
}

}  // namespace sx
