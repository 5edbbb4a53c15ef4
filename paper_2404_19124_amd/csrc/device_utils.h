// Small device helpers: bf16 <-> f32, (value, index) ordering, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specdraft {

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

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
// best (value, index) over the wave; every lane gets the result
__device__ __forceinline__ void wave_best(float& v, int32_t& i) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) {
    float ov = __shfl_xor(v, o, 64);
    int32_t oi = __shfl_xor(i, o, 64);
    if (before(ov, oi, v, i)) { v = ov; i = oi; }
  }
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
