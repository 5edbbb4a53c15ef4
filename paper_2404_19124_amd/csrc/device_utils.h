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
template <int CTRL>
__device__ __forceinline__ void best_step(float& v, int32_t& i) {
  const float ov = dpp_f<CTRL>(v);
  const int32_t oi = dpp_i<CTRL>(i);
  if (before(ov, oi, v, i)) { v = ov; i = oi; }
}
// best (value, index) over each row of 16 lanes
__device__ __forceinline__ void row16_best(float& v, int32_t& i) {
  best_step<kDppXor1>(v, i);
  best_step<kDppXor2>(v, i);
  best_step<kDppHalfMirror>(v, i);
  best_step<kDppMirror>(v, i);
}

__device__ __forceinline__ float wave_sum(float x) {
  x = row16_sum(x);
  return (lane_f(x, 0) + lane_f(x, 16)) + (lane_f(x, 32) + lane_f(x, 48));
}
__device__ __forceinline__ float wave_max(float x) {
  x = row16_max(x);
  return fmaxf(fmaxf(lane_f(x, 0), lane_f(x, 16)), fmaxf(lane_f(x, 32), lane_f(x, 48)));
}
// best (value, index) over the wave; every lane gets the result
__device__ __forceinline__ void wave_best(float& v, int32_t& i) {
  row16_best(v, i);
  float bv = lane_f(v, 0);
  int32_t bi = __builtin_amdgcn_readlane(i, 0);
#pragma unroll
  for (int r = 16; r < 64; r += 16) {
    const float ov = lane_f(v, r);
    const int32_t oi = __builtin_amdgcn_readlane(i, r);
    if (before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
  }
  v = bv;
  i = bi;
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
  wave_best(v, i);
  const int w = threadIdx.x >> 6, nw = NT / 64;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) { sv[w] = v; si[w] = i; }
  __syncthreads();
  v = sv[0];
  i = si[0];
  for (int j = 1; j < nw; ++j)
    if (before(sv[j], si[j], v, i)) { v = sv[j]; i = si[j]; }
}

}  // namespace specdraft
