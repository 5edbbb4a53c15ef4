// Small device helpers: bf16 <-> f32, (value, index) ordering, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specdraft {

// erf by the rational approximation 7.1.26 of Abramowitz and Stegun,
//   erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2),  t = 1 / (1 + p x),  x >= 0,
// absolute error <= 1.5e-7 analytically, 6e-7 evaluated in float32: a dozen
// instructions against the ~60 of the library routine.  The stage kernels are a serial
// chain of a few thousand cycles per workgroup at batch 1, and the library erf was a
// fifth of it; the error is four orders of magnitude below one bf16 ulp of a state.
__device__ __forceinline__ float erf_as(float x) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, ax, 1.0f));
  float p = 1.061405429f;
  p = __builtin_fmaf(p, t, -1.453152027f);
  p = __builtin_fmaf(p, t, 1.421413741f);
  p = __builtin_fmaf(p, t, -0.284496736f);
  p = __builtin_fmaf(p, t, 0.254829592f);
  const float e = __builtin_amdgcn_exp2f(-ax * ax * 1.4426950408889634f);
  const float r = __builtin_fmaf(-p * t, e, 1.0f);
  return copysignf(r, x);
}

// threadIdx.x as a value the optimiser cannot look through: device bodies that are inlined into
// larger kernels derive every per-thread index from it, so that the compiler does not hoist those
// computations and keep dozens of registers alive across the whole kernel.
__device__ __forceinline__ int opaque_tid() {
  int t = threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}


#define SPEC_NEG_INF (-__builtin_huge_valf())
constexpr int32_t kIdxNone = 0x7fffffff;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

// round to nearest, ties to even; NaN stays NaN
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}

// Total order used everywhere a "best" is chosen: larger value first, then
// smaller index.  true when (v1, i1) comes strictly before (v2, i2).
__device__ __forceinline__ bool before(float v1, int32_t i1, float v2, int32_t i2) {
  return (v1 > v2) || (v1 == v2 && i1 < i2);
}

// ---- wave reductions ---------------------------------------------------------
// Within a row of 16 lanes the exchange runs on DPP (quad permutes, then the
// half-row and row mirrors): four steps of a few cycles each instead of LDS
// crossbar shuffles.  The four row results are then read with v_readlane and
// combined uniformly, so every lane ends with the result.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
template <int CTRL>
__device__ __forceinline__ int32_t dpp_i(int32_t x) {
  return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, false);
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7-i inside each 8
constexpr int kDppMirror = 0x140;     // lane i <-> 15-i inside each 16
__device__ __forceinline__ float lane_f(float x, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), l));
}

__device__ __forceinline__ float row16_sum(float x) {
  x += dpp_f<kDppXor1>(x);
  x += dpp_f<kDppXor2>(x);
  x += dpp_f<kDppHalfMirror>(x);
  x += dpp_f<kDppMirror>(x);
  return x;
}
__device__ __forceinline__ float row16_max(float x) {
  x = fmaxf(x, dpp_f<kDppXor1>(x));
  x = fmaxf(x, dpp_f<kDppXor2>(x));
  x = fmaxf(x, dpp_f<kDppHalfMirror>(x));
  x = fmaxf(x, dpp_f<kDppMirror>(x));
  return x;
}
// (value, index) pairs are reduced as ONE 64-bit key: high word = the float mapped to an unsigned
// integer of the same order (zeros of both signs alike, NaN below everything: it never wins, as
// under before()), low word = ~index (smaller index = larger key).  A reduction step is then two
// DPP moves, one 64-bit compare and two selects; compares of the pair in three pieces with the
// mask logic on the scalar unit took twice the instructions and a round trip between the units.
__device__ __forceinline__ uint64_t best_key(float v, int32_t i) {
  const uint32_t u = __float_as_uint(v + 0.0f);
  const uint32_t k = u ^ (static_cast<uint32_t>(static_cast<int32_t>(u) >> 31) | 0x80000000u);
  return (static_cast<uint64_t>(v != v ? 0u : k) << 32) | static_cast<uint32_t>(~i);
}
__device__ __forceinline__ void best_unkey(uint64_t key, float& v, int32_t& i) {
  const uint32_t k = static_cast<uint32_t>(key >> 32);
  v = __uint_as_float((k & 0x80000000u) ? (k ^ 0x80000000u) : ~k);
  i = static_cast<int32_t>(~static_cast<uint32_t>(key));
}
// A key the optimiser cannot look through.  Lists of keys live in registers and move up by one when
// their head is taken ("a[q] = won ? a[q + 1] : a[q]"); left alone, the compiler turns that into
// a[won ? q + 1 : q], a dynamic index into registers, i.e. a chain of selects over the whole list per entry.
__device__ __forceinline__ uint64_t opaque_key(uint64_t x) {
  asm("" : "+v"(x));
  return x;
}
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ uint64_t key_step(uint64_t key) {
  // rows outside ROW_MASK keep their own key (old = source): the step is then a no-op for them
  const int32_t hi = static_cast<int32_t>(key >> 32), lo = static_cast<int32_t>(key);
  const uint32_t oh = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(hi, hi, CTRL, ROW_MASK, 0xf, false));
  const uint32_t ol = static_cast<uint32_t>(__builtin_amdgcn_update_dpp(lo, lo, CTRL, ROW_MASK, 0xf, false));
  const uint64_t other = (static_cast<uint64_t>(oh) << 32) | ol;
  return other > key ? other : key;
}
__device__ __forceinline__ uint64_t row16_best_key(uint64_t key) {
  key = key_step<kDppXor1>(key);
  key = key_step<kDppXor2>(key);
  key = key_step<kDppHalfMirror>(key);
  return key_step<kDppMirror>(key);
}
// best (value, index) over each row of 16 lanes
__device__ __forceinline__ void row16_best(float& v, int32_t& i) {
  best_unkey(row16_best_key(best_key(v, i)), v, i);
}

__device__ __forceinline__ float wave_sum(float x) {
  x = row16_sum(x);
  return (lane_f(x, 0) + lane_f(x, 16)) + (lane_f(x, 32) + lane_f(x, 48));
}
__device__ __forceinline__ float wave_max(float x) {
  x = row16_max(x);
  return fmaxf(fmaxf(lane_f(x, 0), lane_f(x, 16)), fmaxf(lane_f(x, 32), lane_f(x, 48)));
}

// best (value, index) over the wave; every lane gets the result.  The four row results are
// combined on DPP row broadcasts (lane 15 of a row into the next row, then lane 31 into the
// upper half: lane 63 ends with the wave's best) and read back once.
constexpr int kDppRowBcast15 = 0x142;
constexpr int kDppRowBcast31 = 0x143;
// largest key over the wave; every lane gets it
__device__ __forceinline__ uint64_t wave_best_key(uint64_t key) {
  key = row16_best_key(key);
  key = key_step<kDppRowBcast15, 0xa>(key);
  key = key_step<kDppRowBcast31, 0xc>(key);
  const uint32_t hi = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int32_t>(key >> 32), 63));
  const uint32_t lo = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int32_t>(key), 63));
  return (static_cast<uint64_t>(hi) << 32) | lo;
}
__device__ __forceinline__ void wave_best(float& v, int32_t& i) {
  best_unkey(wave_best_key(best_key(v, i)), v, i);
}

// Block-wide helpers for blocks of NT threads (NT multiple of 64, <= 1024).
// `scratch` needs 2 * (NT/64) words; all threads must call.
template <int NT>
__device__ __forceinline__ float block_sum(float x, float* scratch) {
  x = wave_sum(x);
  const int w = threadIdx.x >> 6, nw = NT / 64;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[w] = x;
  __syncthreads();
  float t = 0.f;
  for (int j = 0; j < nw; ++j) t += scratch[j];
  return t;
}
template <int NT>
__device__ __forceinline__ float block_max(float x, float* scratch) {
  x = wave_max(x);
  const int w = threadIdx.x >> 6, nw = NT / 64;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) scratch[w] = x;
  __syncthreads();
  float t = scratch[0];
  for (int j = 1; j < nw; ++j) t = fmaxf(t, scratch[j]);
  return t;
}
template <int NT>
__device__ __forceinline__ void block_best(float& v, int32_t& i, float* sv, int32_t* si) {
  const uint64_t wk = wave_best_key(best_key(v, i));
  const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
  constexpr int nw = NT / 64;
  static_assert(nw <= 16, "the waves' results are combined by one row of 16 lanes");
  __syncthreads();
  if (lane == 0) {
    sv[w] = __uint_as_float(static_cast<uint32_t>(wk >> 32));
    si[w] = static_cast<int32_t>(static_cast<uint32_t>(wk));
  }
  __syncthreads();
  // the waves' keys, one per lane of a 16-lane row, reduced on DPP (every row computes the same)
  const int l16 = lane & 15;
  uint64_t key = 0;   // below every key
  if (l16 < nw) key = (static_cast<uint64_t>(__float_as_uint(sv[l16])) << 32) | static_cast<uint32_t>(si[l16]);
  best_unkey(row16_best_key(key), v, i);
}

}  // namespace specdraft
