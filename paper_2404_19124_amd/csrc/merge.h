// Wave-level merge of the per-part results of a head contraction into the
// row's log-sum-exp and its k best (logit, token) pairs.
#pragma once
#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

// All 64 lanes of a wave call this for the same row; every lane receives the
// result.  out_val / out_idx must be indexed with compile-time constants by the
// caller (they live in registers).  Candidates of different parts never share a
// vocabulary index, so (value, index) is a strict total order.
__device__ __forceinline__ void wave_merge_partials(const Partials& p, int64_t row, int nparts, int k,
                                                    float (&out_val)[kMaxTopK], int32_t (&out_idx)[kMaxTopK],
                                                    float& lse) {
  const int lane = threadIdx.x & 63;
  const float* pm = p.m + row * nparts;
  const float* ps = p.s + row * nparts;
  const float* pv = p.val + row * (int64_t)nparts * k;
  const int32_t* pi = p.idx + row * (int64_t)nparts * k;

  float mx = SPEC_NEG_INF;
  for (int c = lane; c < nparts; c += 64) mx = fmaxf(mx, pm[c]);
  mx = wave_max(mx);
  float sum = 0.f;
  for (int c = lane; c < nparts; c += 64) {
    const float m = pm[c];
    if (m > SPEC_NEG_INF) sum += ps[c] * expf(m - mx);
  }
  sum = wave_sum(sum);
  lse = mx + logf(sum);

  const int total = nparts * k;
  float lastv = __builtin_huge_valf();
  int32_t lasti = -1;
#pragma unroll
  for (int j = 0; j < kMaxTopK; ++j) {
    out_val[j] = SPEC_NEG_INF;
    out_idx[j] = kIdxNone;
    if (j < k) {
      float bv = SPEC_NEG_INF;
      int32_t bi = kIdxNone;
      for (int c = lane; c < total; c += 64) {
        const float v = pv[c];
        const int32_t i = pi[c];
        if (before(lastv, lasti, v, i) && before(v, i, bv, bi)) { bv = v; bi = i; }
      }
      wave_best(bv, bi);
      out_val[j] = bv;
      out_idx[j] = bi;
      lastv = bv;
      lasti = bi;
    }
  }
}

}  // namespace specdraft
