// Wave-level merge of the per-part results of a head contraction into the
// row's log-sum-exp and its k best (logit, token) pairs.
#pragma once
#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

// Insert (v, i) into a list kept sorted by "larger value, then smaller index";
// the last entry falls off.
template <int K>
__device__ __forceinline__ void list_insert(float (&tv)[K], int32_t (&ti)[K], float v, int32_t i) {
  float cv = v;
  int32_t ci = i;
#pragma unroll
  for (int q = 0; q < K; ++q) {
    const bool gt = before(cv, ci, tv[q], ti[q]);
    const float ov = tv[q];
    const int32_t oi = ti[q];
    tv[q] = gt ? cv : ov;
    ti[q] = gt ? ci : oi;
    cv = gt ? ov : cv;
    ci = gt ? oi : ci;
  }
}

// All 64 lanes of a wave call this for the same row; every lane receives the
// result.  out_val / out_idx must be indexed with compile-time constants by the
// caller (they live in registers).  Candidates of different parts never share a
// vocabulary index, so (value, index) is a strict total order.
//
// Latency matters here (this sits on the serial chain between two heads at
// batch 1): every lane first issues the loads of four parts at once, then folds
// them into a sorted register list; the k results are popped with wave-wide
// reductions, no memory traffic in between.
template <int K>
__device__ __forceinline__ void wave_merge_partials_k(const Partials& p, int64_t row, int nparts, int k,
                                                    float (&out_val)[kMaxTopK], int32_t (&out_idx)[kMaxTopK],
                                                    float& lse) {
  const int lane = opaque_tid() & 63;
  const float* pm = p.m + row * nparts;
  const float* ps = p.s + row * nparts;
  const float* pv = p.val + row * (int64_t)nparts * k;
  const int32_t* pi = p.idx + row * (int64_t)nparts * k;

  // the lane's list, as 64-bit keys (best_key): sorted, empty slots hold the key of (-inf, none)
  const uint64_t kEmpty = best_key(SPEC_NEG_INF, kIdxNone);
  uint64_t tk[K];
#pragma unroll
  for (int q = 0; q < K; ++q) tk[q] = kEmpty;
  float run_m = SPEC_NEG_INF, run_s = 0.f;

  constexpr int UN = 4;
  for (int p0 = 0; p0 < nparts; p0 += 64 * UN) {
    float lm[UN], ls[UN], lv[UN][K];
    int32_t li[UN][K];
#pragma unroll
    for (int u = 0; u < UN; ++u) {
      // every load is unconditional (clamped to a valid slot) so that all of them are
      // in flight together; what does not exist is masked after it arrives
      const int part = p0 + u * 64 + lane;
      const bool ok = part < nparts;
      const int pc = ok ? part : nparts - 1;
      const float m_ = pm[pc], s_ = ps[pc];
      lm[u] = ok ? m_ : SPEC_NEG_INF;
      ls[u] = ok ? s_ : 0.f;
#pragma unroll
      for (int j = 0; j < K; ++j) {
        const int jc = j < k ? j : k - 1;
        const float v_ = pv[(int64_t)pc * k + jc];
        const int32_t i_ = pi[(int64_t)pc * k + jc];
        const bool okj = ok && j < k;
        lv[u][j] = okj ? v_ : SPEC_NEG_INF;
        li[u][j] = okj ? i_ : kIdxNone;
      }
    }
    // softmax pieces of this lane's UN parts: one exponential per part (the fast one: its 1e-6
    // relative error is far inside what separates float32 from float64 accumulation)
    float mloc = lm[0];
#pragma unroll
    for (int u = 1; u < UN; ++u) mloc = fmaxf(mloc, lm[u]);
    float sloc = 0.f;
#pragma unroll
    for (int u = 0; u < UN; ++u) sloc += lm[u] > SPEC_NEG_INF ? ls[u] * __expf(lm[u] - mloc) : 0.f;
    if (p0 == 0) {
      run_m = mloc;
      run_s = sloc;
    } else if (mloc > SPEC_NEG_INF) {
      const float mn = fmaxf(run_m, mloc);
      run_s = run_s * __expf(run_m - mn) + sloc * __expf(mloc - mn);
      run_m = mn;
    }
    // branch-free insertion: a chain of compare-exchanges down the list (an entry that does not
    // belong, the empty key included, falls through and changes nothing)
#pragma unroll
    for (int u = 0; u < UN; ++u) {
#pragma unroll
      for (int j = 0; j < K; ++j) {
        uint64_t x = best_key(lv[u][j], li[u][j]);
#pragma unroll
        for (int q = 0; q < K; ++q) {
          const bool gt = x > tk[q];
          const uint64_t lower = gt ? tk[q] : x;
          tk[q] = gt ? x : tk[q];
          x = lower;
        }
      }
    }
  }

  const float mx = wave_max(run_m);
  const float sum = wave_sum(run_m > SPEC_NEG_INF ? run_s * __expf(run_m - mx) : 0.f);
  lse = mx + logf(sum);

#pragma unroll
  for (int j = 0; j < kMaxTopK; ++j) {
    out_val[j] = SPEC_NEG_INF;
    out_idx[j] = kIdxNone;
  }
#pragma unroll
  for (int j = 0; j < K; ++j) {
    if (j < k) {
      const uint64_t best = wave_best_key(tk[0]);
      const bool won = tk[0] == best;   // the owner of the winner pops it (keys of real entries are unique)
#pragma unroll
      for (int q = 0; q + 1 < K; ++q) {
        const uint64_t up = opaque_key(tk[q + 1]);
        tk[q] = won ? up : tk[q];
      }
      tk[K - 1] = won ? kEmpty : tk[K - 1];
      best_unkey(best, out_val[j], out_idx[j]);
    }
  }
}

// The same merge done by a group of 256 consecutive threads for ONE row: with at most
// 256 parts every thread holds exactly one part's (already sorted) list, so nothing has
// to be inserted.  Two levels, ONE exchange: every wave reduces its 64 parts to its own
// (max, sum-exp, k best) with wave-wide reductions only, the four waves' results go
// through LDS behind a single barrier, and every thread merges the four sorted lists.
// (A pop per round across the whole group - one barrier and one LDS exchange per result -
// took 0.65 us per round on the batch-1 chain.)  A workgroup of 256 * n threads runs n such
// groups side by side (each on its own row, or all on the same one): the function contains
// workgroup barriers, so EVERY thread of the workgroup must call it, with the same k
// and nparts; every thread receives its group's result.  `lds` is the group's own
// scratch of kMergeLds words.
constexpr int kMergeWave = 2 + 2 * kMaxTopK;   // words per wave: max, sum-exp, k values, k indices
constexpr int kMergeLds = 4 * kMergeWave;
template <int K>
__device__ __forceinline__ void group_merge_partials_k(const Partials& p, int64_t row, int nparts, int k,
                                                     float (&out_val)[kMaxTopK], int32_t (&out_idx)[kMaxTopK],
                                                     float& lse, float* lds) {
  const int gt = opaque_tid() & 255, lane = gt & 63, w = gt >> 6;
  const float* pm = p.m + row * nparts;
  const float* ps = p.s + row * nparts;
  const float* pv = p.val + row * (int64_t)nparts * k;
  const int32_t* pi = p.idx + row * (int64_t)nparts * k;

  float tv[K];
  int32_t ti[K];
  float run_m = SPEC_NEG_INF, run_s = 0.f;
  {
    const bool ok = gt < nparts;
    const int pc = ok ? gt : nparts - 1;
    const float m_ = pm[pc], s_ = ps[pc];
#pragma unroll
    for (int j = 0; j < K; ++j) {
      const int jc = j < k ? j : k - 1;
      const float v_ = pv[(int64_t)pc * k + jc];
      const int32_t i_ = pi[(int64_t)pc * k + jc];
      const bool okj = ok && j < k;
      tv[j] = okj ? v_ : SPEC_NEG_INF;
      ti[j] = okj ? i_ : kIdxNone;
    }
    if (ok) { run_m = m_; run_s = s_; }
  }
  for (int part = gt + 256; part < nparts; part += 256) {   // more parts than threads: fold the rest in
    const float m_ = pm[part], s_ = ps[part];
    if (m_ > SPEC_NEG_INF) {
      const float mn = fmaxf(run_m, m_);
      run_s = run_s * __expf(run_m - mn) + s_ * __expf(m_ - mn);
      run_m = mn;
    }
    for (int j = 0; j < k; ++j) {
      const float v_ = pv[(int64_t)part * k + j];
      const int32_t i_ = pi[(int64_t)part * k + j];
      if (before(v_, i_, tv[K - 1], ti[K - 1])) list_insert<K>(tv, ti, v_, i_);
    }
  }

  // ---- this wave's 64 parts
  const float wm = wave_max(run_m);
  const float wsum = wave_sum(run_m > SPEC_NEG_INF ? run_s * __expf(run_m - wm) : 0.f);
  float wv[K];
  int32_t wi[K];
#pragma unroll
  for (int j = 0; j < K; ++j) {
    wv[j] = SPEC_NEG_INF;
    wi[j] = kIdxNone;
    if (j < k) {
      float bv = tv[0];
      int32_t bi = ti[0];
      wave_best(bv, bi);
      if (ti[0] == bi && tv[0] == bv) {  // the owner of the winner pops it
#pragma unroll
        for (int q = 0; q + 1 < K; ++q) { tv[q] = tv[q + 1]; ti[q] = ti[q + 1]; }
        tv[K - 1] = SPEC_NEG_INF;
        ti[K - 1] = kIdxNone;
      }
      wv[j] = bv;
      wi[j] = bi;
    }
  }

  // ---- the four waves' results through LDS
  float* mine = lds + w * kMergeWave;
  __syncthreads();                                    // scratch may still be read from an earlier call
  if (lane == 0) {
    mine[0] = wm;
    mine[1] = wsum;
#pragma unroll
    for (int j = 0; j < K; ++j) {
      mine[2 + j] = wv[j];
      reinterpret_cast<int32_t*>(mine)[2 + kMaxTopK + j] = wi[j];
    }
  }
  __syncthreads();
  float m4[4], s4[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) { m4[q] = lds[q * kMergeWave]; s4[q] = lds[q * kMergeWave + 1]; }
  const float mx = fmaxf(fmaxf(m4[0], m4[1]), fmaxf(m4[2], m4[3]));
  float sum = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q) sum += m4[q] > SPEC_NEG_INF ? s4[q] * __expf(m4[q] - mx) : 0.f;
  lse = mx + logf(sum);

#pragma unroll
  for (int j = 0; j < kMaxTopK; ++j) {
    out_val[j] = SPEC_NEG_INF;
    out_idx[j] = kIdxNone;
  }
  // four sorted lists, as 64-bit keys in registers (one batch of LDS reads): only their heads compete;
  // the list whose head won moves up by one (keys are unique: every candidate has its own token)
  uint64_t lk[4][K];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int t = 0; t < K; ++t)
      lk[q][t] = best_key(lds[q * kMergeWave + 2 + t],
                          reinterpret_cast<const int32_t*>(lds)[q * kMergeWave + 2 + kMaxTopK + t]);
#pragma unroll
  for (int j = 0; j < K; ++j) {
    if (j < k) {
      uint64_t best = lk[0][0];
#pragma unroll
      for (int q = 1; q < 4; ++q) best = lk[q][0] > best ? lk[q][0] : best;
      best_unkey(best, out_val[j], out_idx[j]);
      if (j + 1 < k) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bool won = lk[q][0] == best;
#pragma unroll
          for (int t = 0; t + 1 < K; ++t) lk[q][t] = won ? lk[q][t + 1] : lk[q][t];
          lk[q][K - 1] = won ? best_key(SPEC_NEG_INF, kIdxNone) : lk[q][K - 1];
        }
      }
    }
  }
}

__device__ __forceinline__ void group_merge_partials(const Partials& p, int64_t row, int nparts, int k,
                                                     float (&out_val)[kMaxTopK], int32_t (&out_idx)[kMaxTopK],
                                                     float& lse, float* lds) {
  switch (k) {
    case 1: group_merge_partials_k<1>(p, row, nparts, k, out_val, out_idx, lse, lds); break;
    case 2: group_merge_partials_k<2>(p, row, nparts, k, out_val, out_idx, lse, lds); break;
    case 3: group_merge_partials_k<3>(p, row, nparts, k, out_val, out_idx, lse, lds); break;
    case 4: group_merge_partials_k<4>(p, row, nparts, k, out_val, out_idx, lse, lds); break;
    case 5:
    case 6: group_merge_partials_k<6>(p, row, nparts, k, out_val, out_idx, lse, lds); break;
    default: group_merge_partials_k<8>(p, row, nparts, k, out_val, out_idx, lse, lds); break;
  }
}

// k is uniform over the launch: pick the list size that just holds it, so that
// the common narrow heads (k = 1..3) do not pay for eight slots.
__device__ __forceinline__ void wave_merge_partials(const Partials& p, int64_t row, int nparts, int k,
                                                    float (&out_val)[kMaxTopK], int32_t (&out_idx)[kMaxTopK],
                                                    float& lse) {
  switch (k) {
    case 1: wave_merge_partials_k<1>(p, row, nparts, k, out_val, out_idx, lse); break;
    case 2: wave_merge_partials_k<2>(p, row, nparts, k, out_val, out_idx, lse); break;
    case 3: wave_merge_partials_k<3>(p, row, nparts, k, out_val, out_idx, lse); break;
    case 4: wave_merge_partials_k<4>(p, row, nparts, k, out_val, out_idx, lse); break;
    case 5:
    case 6: wave_merge_partials_k<6>(p, row, nparts, k, out_val, out_idx, lse); break;
    default: wave_merge_partials_k<8>(p, row, nparts, k, out_val, out_idx, lse); break;
  }
}

}  // namespace specdraft
