// Verification (Sec. 1, 3.1, 5 of the paper), greedy:
//   greedy[b,c,p]  = first maximum of base_logits[b,c,p,:]
//   accept[b,c]    = number of leading positions p with greedy[b,c,p] == cand[b,c,p]
//   best[b]        = first candidate with the longest accepted prefix
//   out            = cand[b,best,:a] ++ greedy[b,best,a]   (the bonus token)
// The row scan is the only part that touches real memory: one workgroup (NT threads) per
// (b,c,p) row, 16-byte loads, (value, index) reduced with "larger value, then
// smaller index".
#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

template <bool BF16, bool VEC, int NT>
__global__ __launch_bounds__(NT) void argmax_rows_kernel(const void* logits, int V, int B, int n1,
                                                           const int32_t* n_cand, int32_t* greedy) {
  __shared__ float sv[16];
  __shared__ int32_t si[16];
  const int64_t row = blockIdx.x;
  const int tid = threadIdx.x;
  if (n_cand) {
    // per-sequence candidate counts: rows of padding candidates are not read at all
    const int p = (int)(row % n1);
    const int64_t qc = row / n1;
    const int c = (int)(qc % B), nc = n_cand[qc / B];
    if (c >= max(nc, 1) || (nc == 0 && p > 0)) {
      if (tid == 0) greedy[row] = -1;
      return;
    }
  }
  // (a thread meets its elements in increasing index order, so a strict "larger" keeps the first maximum;
  // the (value, smaller index) order only matters between threads)
  float bv = SPEC_NEG_INF;
  int32_t bi = kIdxNone;
  if (BF16) {
    const uint16_t* x = static_cast<const uint16_t*>(logits) + row * V;
    if (VEC) {
      // (non-temporal: the logits are read once; a stream that does not allocate in the
      // caches is the faster one on this chip)
      // eight loads in flight per thread: at small batch the kernel is a chain of memory
      // round trips, not a stream
      const u32x4* xv = reinterpret_cast<const u32x4*>(x);
      const int nvec = V / 8;
      constexpr int U = 8192 / NT;
      for (int c0 = tid; c0 < nvec; c0 += NT * U) {
        u32x4 raw[U];
#pragma unroll
        for (int u = 0; u < U; ++u) raw[u] = __builtin_nontemporal_load(xv + min(c0 + u * NT, nvec - 1));
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int c = c0 + u * NT;
          if (c < nvec) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const float lo = bf16_bits_to_f32(raw[u][q] & 0xffffu), hi = bf16_bits_to_f32(raw[u][q] >> 16);
              const int i0 = c * 8 + 2 * q;
              if (lo > bv) { bv = lo; bi = i0; }
              if (hi > bv) { bv = hi; bi = i0 + 1; }
            }
          }
        }
      }
      for (int i = (V / 8) * 8 + tid; i < V; i += NT) {
        const float v = bf16_bits_to_f32(x[i]);
        if (v > bv) { bv = v; bi = i; }
      }
    } else {
      for (int i = tid; i < V; i += NT) {
        const float v = bf16_bits_to_f32(x[i]);
        if (v > bv) { bv = v; bi = i; }
      }
    }
  } else {
    const float* x = static_cast<const float*>(logits) + row * V;
    if (VEC) {
      const f32x4* xv = reinterpret_cast<const f32x4*>(x);
      const int nvec = V / 4;
      constexpr int U = 8192 / NT;
      for (int c0 = tid; c0 < nvec; c0 += NT * U) {
        f32x4 r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) r[u] = __builtin_nontemporal_load(xv + min(c0 + u * NT, nvec - 1));
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int c = c0 + u * NT;
          if (c < nvec) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (r[u][q] > bv) { bv = r[u][q]; bi = c * 4 + q; }
          }
        }
      }
      for (int i = (V / 4) * 4 + tid; i < V; i += NT) {
        const float v = x[i];
        if (v > bv) { bv = v; bi = i; }
      }
    } else {
      for (int i = tid; i < V; i += NT) {
        const float v = x[i];
        if (v > bv) { bv = v; bi = i; }
      }
    }
  }
  block_best<NT>(bv, bi, sv, si);
  // a row of NaNs (or of -inf) has no "larger" element: report index 0 like a first-maximum scan
  if (tid == 0) greedy[row] = (bi == kIdxNone) ? 0 : bi;
}

hipError_t launch_argmax_rows(const void* logits, int bf16, int64_t rows, int V, int B, int n1, const int32_t* n_cand,
                              int32_t* greedy, hipStream_t st) {
  const size_t esz = bf16 ? 2 : 4;
  // 16-byte loads need every row to start on a 16-byte boundary
  const bool vec = ((size_t)V * esz) % 16 == 0 && (reinterpret_cast<uintptr_t>(logits) % 16) == 0;
  dim3 grid((unsigned)rows);
  // a few rows (small batch): a chain of memory round trips, the more loads in flight per row the better;
  // thousands of rows: a stream, which runs a little faster from 512-thread workgroups (7B batch 64: 81 -> 79.4 us)
  const int nt = rows >= 1024 ? 512 : 1024;
#define LAUNCH_ARGMAX(B16, VEC, NT) \
  hipLaunchKernelGGL((argmax_rows_kernel<B16, VEC, NT>), grid, dim3(NT), 0, st, logits, V, B, n1, n_cand, greedy)
#define LAUNCH_ARGMAX_NT(B16, VEC) \
  do { if (nt == 512) LAUNCH_ARGMAX(B16, VEC, 512); else LAUNCH_ARGMAX(B16, VEC, 1024); } while (0)
  if (bf16) {
    if (vec) LAUNCH_ARGMAX_NT(true, true); else LAUNCH_ARGMAX_NT(true, false);
  } else {
    if (vec) LAUNCH_ARGMAX_NT(false, true); else LAUNCH_ARGMAX_NT(false, false);
  }
  return hipGetLastError();
}

__global__ __launch_bounds__(64) void accept_kernel(const int32_t* greedy, const int32_t* cand, const int32_t* n_cand,
                                                    int B, int n, int32_t* accept_len, int32_t* best_cand,
                                                    int32_t* out_tokens, int32_t* n_out, int32_t* accept_all) {
  const int q = blockIdx.x, lane = threadIdx.x;
  // candidates of this sequence (the rest of its B slots is padding); none = speculation off: the
  // first slot stands for the empty candidate, whose accepted length is 0
  const int nc = n_cand ? n_cand[q] : B;
  // (accepted length, candidate): longer first, then smaller candidate index
  float bv = -1.f;
  int32_t bi = kIdxNone;
  for (int c = lane; c < B; c += 64) {
    const int32_t* g = greedy + ((int64_t)q * B + c) * (n + 1);
    const int32_t* t = cand + ((int64_t)q * B + c) * n;
    // all positions are requested at once (one round trip, not one per accepted token)
    int32_t gg[kMaxStages], tt[kMaxStages];
#pragma unroll
    for (int p = 0; p < kMaxStages; ++p) {
      gg[p] = p < n ? g[p] : 0;
      tt[p] = p < n ? t[p] : -1;
    }
    int a = 0;
    bool run = c < nc;
#pragma unroll
    for (int p = 0; p < kMaxStages; ++p) {
      run = run && p < n && gg[p] == tt[p];
      a += run ? 1 : 0;
    }
    if (accept_all) accept_all[(int64_t)q * B + c] = a;
    if (c < max(nc, 1) && before((float)a, c, bv, bi)) { bv = (float)a; bi = c; }
  }
  wave_best(bv, bi);
  const int a = (int)bv, best = bi;
  if (lane == 0) {
    accept_len[q] = a;
    best_cand[q] = best;
    n_out[q] = a + 1;
  }
  const int32_t* g = greedy + ((int64_t)q * B + best) * (n + 1);
  const int32_t* t = cand + ((int64_t)q * B + best) * n;
  for (int p = lane; p <= n; p += 64) out_tokens[(int64_t)q * (n + 1) + p] = p < a ? t[p] : (p == a ? g[a] : -1);
}

hipError_t launch_accept(const int32_t* greedy, const int32_t* cand, const int32_t* n_cand, int batch, int B, int n,
                         int32_t* accept_len, int32_t* best_cand, int32_t* out_tokens, int32_t* n_out,
                         int32_t* accept_all, hipStream_t st) {
  hipLaunchKernelGGL(accept_kernel, dim3(batch), dim3(64), 0, st, greedy, cand, n_cand, B, n, accept_len, best_cand,
                     out_tokens, n_out, accept_all);
  return hipGetLastError();
}

}  // namespace specdraft
