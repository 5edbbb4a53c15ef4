// float32 path (the small correctness configuration keeps every tensor in
// float32 with no rounding anywhere) and the bf16 tiling kernel.
// The float32 contraction is a plain LDS-tiled vector-ALU kernel: this path is
// there for exactness on small shapes, not for speed; logits are materialised in
// a workspace and reduced per row.
#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

// ---- tiling of a row-major bf16 matrix into matrix-core fragment order -------
__global__ __launch_bounds__(256) void pack_bf16_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                        int n_rows, int kt, int64_t n_slots, int zero_pad) {
  const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (slot >= n_slots) return;
  const int lane = (int)(slot & 63);
  const int64_t frag = slot >> 6;
  const int t = (int)(frag % kt);
  const int64_t nt = frag / kt;
  const int64_t row = nt * 16 + (lane & 15);
  if (row < n_rows) {
    dst[slot] = src[row * (kt * 4) + t * 4 + (lane >> 4)];   // 8 bf16 = one 16-byte unit
  } else if (zero_pad) {
    dst[slot] = make_uint4(0, 0, 0, 0);
  }
}

hipError_t launch_pack_bf16(const void* src, void* dst, int n_rows, int k, bool zero_pad, hipStream_t st) {
  const int kt = k / 32;
  const int64_t n_slots = (int64_t)((n_rows + 15) / 16) * kt * 64;
  const unsigned grid = (unsigned)((n_slots + 255) / 256);
  hipLaunchKernelGGL(pack_bf16_kernel, dim3(grid), dim3(256), 0, st, static_cast<const uint4*>(src),
                     static_cast<uint4*>(dst), n_rows, kt, n_slots, zero_pad ? 1 : 0);
  return hipGetLastError();
}

// ---- out[r][v] = sum_k a[r][k] * w[v][k] -------------------------------------
constexpr int TM = 32, TN = 64, TK = 16;
__global__ __launch_bounds__(256) void gemm_f32_kernel(const float* __restrict__ a, int64_t lda,
                                                       const float* __restrict__ w, int64_t ldw,
                                                       float* __restrict__ out, int64_t ldo, int R, int N, int K) {
  __shared__ float sa[TK][TM + 1];
  __shared__ float sw[TK][TN + 1];
  const int tid = threadIdx.x;
  const int r0 = blockIdx.y * TM, v0 = blockIdx.x * TN;
  const int tr = tid / 16, tv = tid % 16;  // thread computes rows tr*2..+1, cols tv*4..+3
  float acc[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int i = tid; i < TM * TK; i += 256) {
      const int rr = i / TK, kk = i % TK;
      sa[kk][rr] = (r0 + rr < R && k0 + kk < K) ? a[(int64_t)(r0 + rr) * lda + k0 + kk] : 0.f;
    }
    for (int i = tid; i < TN * TK; i += 256) {
      const int vv = i / TK, kk = i % TK;
      sw[kk][vv] = (v0 + vv < N && k0 + kk < K) ? w[(int64_t)(v0 + vv) * ldw + k0 + kk] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[2], wv[4];
#pragma unroll
      for (int i = 0; i < 2; ++i) av[i] = sa[kk][tr * 2 + i];
#pragma unroll
      for (int q = 0; q < 4; ++q) wv[q] = sw[kk][tv * 4 + q];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[i][q] += av[i] * wv[q];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int r = r0 + tr * 2 + i, v = v0 + tv * 4 + q;
      if (r < R && v < N) out[(int64_t)r * ldo + v] = acc[i][q];
    }
}

hipError_t launch_gemm_f32(const float* a, int64_t lda, const float* w, int64_t ldw, float* out, int64_t ldo, int R,
                           int N, int K, hipStream_t st) {
  dim3 grid((N + TN - 1) / TN, (R + TM - 1) / TM);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, a, lda, w, ldw, out, ldo, R, N, K);
  return hipGetLastError();
}

// ---- one partial (max, sum-exp, k best) per row of materialised logits -------
__global__ __launch_bounds__(256) void row_topk_f32_kernel(const float* __restrict__ logits, int64_t ld, int V,
                                                           int k_top, Partials part) {
  __shared__ float sv[4];
  __shared__ int32_t si[4];
  __shared__ float scratch[8];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  const float* x = logits + row * ld;
  float lastv = __builtin_huge_valf();
  int32_t lasti = -1;
  float mx = 0.f;
  for (int j = 0; j < k_top; ++j) {
    float bv = SPEC_NEG_INF;
    int32_t bi = kIdxNone;
    for (int i = tid; i < V; i += 256) {
      const float v = x[i];
      if (before(lastv, lasti, v, i) && before(v, i, bv, bi)) { bv = v; bi = i; }
    }
    block_best<256>(bv, bi, sv, si);
    if (tid == 0) {
      part.val[row * k_top + j] = bv;
      part.idx[row * k_top + j] = bi;
    }
    if (j == 0) mx = bv;
    lastv = bv;
    lasti = bi;
  }
  float s = 0.f;
  for (int i = tid; i < V; i += 256) s += expf(x[i] - mx);
  s = block_sum<256>(s, scratch);
  if (tid == 0) {
    part.m[row] = mx;
    part.s[row] = s;
  }
}

hipError_t launch_row_topk_f32(const float* logits, int64_t ld, int R, int V, int k_top, Partials part,
                               hipStream_t st) {
  hipLaunchKernelGGL(row_topk_f32_kernel, dim3(R), dim3(256), 0, st, logits, ld, V, k_top, part);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void row_log_softmax_kernel(const float* __restrict__ logits,
                                                              float* __restrict__ logp, int64_t ld, int V) {
  __shared__ float scratch[8];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  const float* x = logits + row * ld;
  float mx = SPEC_NEG_INF;
  for (int i = tid; i < V; i += 256) mx = fmaxf(mx, x[i]);
  mx = block_max<256>(mx, scratch);
  float s = 0.f;
  for (int i = tid; i < V; i += 256) s += expf(x[i] - mx);
  s = block_sum<256>(s, scratch);
  const float lse = mx + logf(s);
  float* y = logp + row * ld;
  for (int i = tid; i < V; i += 256) y[i] = x[i] - lse;
}

hipError_t launch_row_log_softmax(const float* logits, float* logp, int64_t ld, int R, int V, hipStream_t st) {
  hipLaunchKernelGGL(row_log_softmax_kernel, dim3(R), dim3(256), 0, st, logits, logp, ld, V);
  return hipGetLastError();
}

// Plain copy of n 16-byte words, grid-stride: a launch whose HBM traffic is known
// exactly (n * 16 bytes read, n * 16 written), used to calibrate traffic counters.
__global__ __launch_bounds__(256) void copy_probe_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst,
                                                         int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_copy_probe(const void* src, void* dst, int64_t n16, hipStream_t st) {
  const int64_t want = (n16 + 255) / 256;
  const int grid = (int)(want < 1 ? 1 : (want > 16384 ? 16384 : want));
  hipLaunchKernelGGL(copy_probe_kernel, dim3(grid), dim3(256), 0, st, static_cast<const u32x4*>(src),
                     static_cast<u32x4*>(dst), n16);
  return hipGetLastError();
}

}  // namespace specdraft
