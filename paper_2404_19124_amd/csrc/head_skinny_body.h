// Device-side body of the rows <= 16 contraction (vocabulary head and/or a projection
// against at most 16 state rows).  See kernels_head_skinny.hip for the design.
#pragma once
#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

constexpr int kSkinnyWaves = 16;
constexpr int kSkinnySteps = 16;              // max K-steps (of 32) per wave -> K <= 8192
constexpr size_t kSkinnyLdsB = 128 * 1024;    // bytes available for the states
constexpr size_t kSkinnyLdsP = 2 * kSkinnyWaves * 64 * 16;  // partial accumulators, double-buffered


// Dynamic LDS a workgroup needs for R rows of kt 32-wide K steps.
__host__ __device__ inline size_t skinny_state_bytes(int R, int kt) {
  return ((size_t)kt * 4 * R * 16 + 255) & ~(size_t)255;
}

// NS = K-steps per wave held per tile, DEPTH = tiles in flight per wave.
// EXACT: every wave has exactly NS steps (K = 16 * 32 * NS); otherwise waves
// take ceil(kt/16) <= NS steps with the tail predicated off.
//
// The weights are read with non-temporal loads: each byte is used once per launch, and a
// step streams several times the capacity of every cache; measured on MI355X, a stream
// that does not allocate in the caches runs about 12 % faster than one that does.
//
// skinny_prefetch requests the first DEPTH tiles of workgroup `wg` (of G) into the
// register ring; skinny_run consumes the ring (it must have been filled by
// skinny_prefetch with the same arguments), streams the remaining tiles and writes the
// workgroup's results.  Weights are read-only for the whole launch, so the prefetch may
// be issued long before the states exist.
template <int NS, int DEPTH, bool EXACT>
__device__ __forceinline__ void skinny_prefetch(const HeadJob& p, int wg, int G, u32x4 (&a)[DEPTH][NS]) {
  const int kt = p.kt;
  const int tid = opaque_tid(), lane = tid & 63, w = tid >> 6;
  const int spw = EXACT ? NS : (kt + kSkinnyWaves - 1) / kSkinnyWaves;
  const int s0 = min(w * spw, kt);
  const int ns = EXACT ? NS : min(kt, s0 + spw) - s0;
  const int total = p.vt_head + p.vt_proj;
  const u32x4* wh = static_cast<const u32x4*>(p.w_head);
  const u32x4* wp = static_cast<const u32x4*>(p.w_proj);
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
    const int tile = wg + d * G;
    if (tile < total) {
      const u32x4* base =
          tile < p.vt_head ? wh + (int64_t)tile * kt * 64 : wp + (int64_t)(tile - p.vt_head) * kt * 64;
      const u32x4* ptr = base + (int64_t)s0 * 64 + lane;
#pragma unroll
      for (int t = 0; t < NS; ++t)
        if (EXACT || t < ns) a[d][t] = __builtin_nontemporal_load(ptr + t * 64);
    }
  }
}

// The folded first stage (FoldJob): rows of D / 8 eight-element chunks, one chunk per thread,
// NT / (D / 8) rows at a time (the host folds only what fits one round); D is a multiple of 512,
// so a wave never straddles two rows.  Writes the bf16
// states into the kernel's LDS layout (slot tg * R + n = row n, columns 8 tg .. 8 tg + 8).
// `red`: 64 floats of LDS scratch.  Contains workgroup barriers.
template <int NT>
__device__ __forceinline__ void fold_states(const HeadJob& p, u32x4* ldsB, float* red) {
  const FoldJob& f = p.fold;
  const int tid = opaque_tid(), lane = tid & 63, w = tid >> 6;
  const int R = p.R, D = f.D, nchunk = D / 8, wpr = nchunk / 64;
  const int rp = NT / nchunk;  // rows per round
  const int sub = tid / nchunk, c = tid - sub * nchunk;
  int buf = 0;
  for (int r0 = 0; r0 < R; r0 += rp) {
    const int r = r0 + sub;
    const bool live = sub < rp && r < R;
    float z[8], ga[8], be[8];
    float lsum = 0.f;
    if (live) {
      const float* pz = f.pz + (int64_t)r * D + c * 8;
      float4 p0 = *reinterpret_cast<const float4*>(pz);
      float4 p1 = *reinterpret_cast<const float4*>(pz + 4);
      for (int q = 1; q < f.pz_parts; ++q) {
        const float4 q0 = *reinterpret_cast<const float4*>(pz + q * f.pz_part_stride);
        const float4 q1 = *reinterpret_cast<const float4*>(pz + q * f.pz_part_stride + 4);
        p0.x += q0.x; p0.y += q0.y; p0.z += q0.z; p0.w += q0.w;
        p1.x += q1.x; p1.y += q1.y; p1.z += q1.z; p1.w += q1.w;
      }
      const int tok = min(max(f.tok[r], 0), f.V - 1);
      const uint4 raw = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(f.emb) + (int64_t)tok * D + c * 8);
      const float4 g0 = *reinterpret_cast<const float4*>(f.gamma + c * 8);
      const float4 g1 = *reinterpret_cast<const float4*>(f.gamma + c * 8 + 4);
      const float4 b0 = *reinterpret_cast<const float4*>(f.beta + c * 8);
      const float4 b1 = *reinterpret_cast<const float4*>(f.beta + c * 8 + 4);
      ga[0] = g0.x; ga[1] = g0.y; ga[2] = g0.z; ga[3] = g0.w; ga[4] = g1.x; ga[5] = g1.y; ga[6] = g1.z; ga[7] = g1.w;
      be[0] = b0.x; be[1] = b0.y; be[2] = b0.z; be[3] = b0.w; be[4] = b1.x; be[5] = b1.y; be[6] = b1.z; be[7] = b1.w;
      const float pzv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
      const uint32_t ew[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float e = bf16_bits_to_f32((q & 1) ? (ew[q >> 1] >> 16) : (ew[q >> 1] & 0xffffu));
        z[q] = f.w_s * pzv[q] + f.w_e * e;
        lsum += z[q];
      }
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q) { z[q] = 0.f; ga[q] = 0.f; be[q] = 0.f; }
    }
    // per-row sums over the row's wpr waves (two scratch areas per round, two rounds alternate)
    float* ra = red + buf * 32;
    float s = wave_sum(lsum);
    if (lane == 0) ra[w] = s;
    __syncthreads();
    float mean = 0.f;
    for (int q = 0; q < wpr; ++q) mean += ra[min(sub, rp - 1) * wpr + q];
    mean /= (float)D;
    float lvar = 0.f;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const float d = z[q] - mean;
      lvar += live ? d * d : 0.f;
    }
    s = wave_sum(lvar);
    if (lane == 0) ra[16 + w] = s;
    __syncthreads();
    float var = 0.f;
    for (int q = 0; q < wpr; ++q) var += ra[16 + min(sub, rp - 1) * wpr + q];
    var /= (float)D;
    const float rstd = 1.0f / sqrtf(var + f.eps);
    if (live) {
      float sv[8];
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const float y = (z[q] - mean) * rstd * ga[q] + be[q];
        sv[q] = 0.5f * y * (1.0f + erf_as(y * 0.70710678118654752440f));
      }
      u32x4 o;
#pragma unroll
      for (int q = 0; q < 4; ++q) o[q] = f32_to_bf16_bits(sv[2 * q]) | (f32_to_bf16_bits(sv[2 * q + 1]) << 16);
      ldsB[c * R + r] = o;
    }
    buf ^= 1;
  }
}

template <int NS, int DEPTH, bool EXACT>
__device__ __forceinline__ void skinny_run(const HeadJob& p, int wg, int G, u32x4 (&a)[DEPTH][NS],
                                           unsigned char* smem) {
  const int kt = p.kt, R = p.R;
  u32x4* ldsB = reinterpret_cast<u32x4*>(smem);  // [kt][4][R] slots of 8 bf16
  const size_t bytesB = ((size_t)kt * 4 * R * 16 + 255) & ~(size_t)255;
  f32x4* ldsP = reinterpret_cast<f32x4*>(smem + bytesB);  // [2][waves][64]
  const int tid = opaque_tid(), lane = tid & 63, w = tid >> 6;
  constexpr int NT = kSkinnyWaves * 64;

  // ---- this wave's slice of K
  const int spw = EXACT ? NS : (kt + kSkinnyWaves - 1) / kSkinnyWaves;
  const int s0 = min(w * spw, kt);
  const int ns = EXACT ? NS : min(kt, s0 + spw) - s0;
  const int g = lane >> 4, nn = min(lane & 15, R - 1);
  const u32x4* bptr = ldsB + ((int64_t)s0 * 4 + g) * R + nn;  // step t: + t*4*R
  const int total = p.vt_head + p.vt_proj;
  const u32x4* wh = static_cast<const u32x4*>(p.w_head);
  const u32x4* wp = static_cast<const u32x4*>(p.w_proj);
  auto tile_ptr = [&](int tile) -> const u32x4* {
    const u32x4* base = tile < p.vt_head ? wh + (int64_t)tile * kt * 64 : wp + (int64_t)(tile - p.vt_head) * kt * 64;
    return base + (int64_t)s0 * 64 + lane;
  };

  // ---- states -> LDS, trimmed to R rows: slot (t, g, n) = row n, columns t*32 + g*8 .. +8
  if (p.fold.enabled) {
    fold_states<NT>(p, ldsB, reinterpret_cast<float*>(ldsP));
  } else if (p.b_rowmajor) {
    for (int n = 0; n < R; ++n) {
      const uint16_t* row = static_cast<const uint16_t*>(p.b_src) + (int64_t)n * p.b_ld;
      for (int tg = tid; tg < kt * 4; tg += NT) ldsB[tg * R + n] = *reinterpret_cast<const u32x4*>(row + tg * 8);
    }
  } else {
    // walk the tiled source linearly: source slot s holds row s%16 of column group s/16
    const u32x4* src = static_cast<const u32x4*>(p.b_src);
#pragma unroll 4
    for (int s = tid; s < kt * 64; s += NT) {
      const int n = s & 15;
      if (n < R) ldsB[(s >> 4) * R + n] = src[s];
    }
  }
  __syncthreads();

  // running state of the 256 epilogue threads: state row en, vocabulary residue vi
  // (16 consecutive threads own one state row: the closing merge of a row's 16 residue lists then runs on
  // DPP alone, no transposition through LDS; the price is a 4-way bank conflict on the 16 partial-sum
  // reads per tile, a few hundred LDS cycles in a tile of several thousand)
  const int en = (tid >> 4) & 15, vi = tid & 15;
  float run_m = SPEC_NEG_INF, run_s = 0.f;
  float tv[kMaxTopK];
  int32_t ti[kMaxTopK];
#pragma unroll
  for (int q = 0; q < kMaxTopK; ++q) { tv[q] = SPEC_NEG_INF; ti[q] = kIdxNone; }

  int buf = 0;
  for (int base = wg; base < total; base += DEPTH * G) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int tile = base + d * G;
      if (tile < total) {
        const int next = tile + DEPTH * G;
        const bool has_next = next < total;
        const u32x4* nptr = tile_ptr(has_next ? next : tile);
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < NS; ++t) {
          if (EXACT || t < ns) {
            const u32x4 b = bptr[(int64_t)t * 4 * R];
            acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[d][t]),
                                                          __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
            if (has_next) a[d][t] = __builtin_nontemporal_load(nptr + t * 64);
          }
        }
        ldsP[(buf * kSkinnyWaves + w) * 64 + lane] = acc;
        __syncthreads();
        if (tid < 256) {
          // accumulator lane l holds state row l%16 and weight rows (l/16)*4 + i
          const float* P = reinterpret_cast<const float*>(ldsP + buf * kSkinnyWaves * 64);
          const int l = (vi >> 2) * 16 + en, i = vi & 3;
          float sum = 0.f;
#pragma unroll
          for (int ww = 0; ww < kSkinnyWaves; ++ww) sum += P[(ww * 64 + l) * 4 + i];
          if (en < R) {
            if (tile < p.vt_head) {
              const int v = tile * 16 + vi;
              if (v < p.n_head) {
                if (p.out_head) {
                  p.out_head[(int64_t)en * p.ld_head + v] = sum;
                } else {
                  const float m_new = fmaxf(run_m, sum);
                  run_s = run_s * __expf(run_m - m_new) + __expf(sum - m_new);
                  run_m = m_new;
                  if (sum > tv[kMaxTopK - 1]) {
                    float cv = sum;
                    int32_t ci = v;
#pragma unroll
                    for (int q = 0; q < kMaxTopK; ++q) {
                      const bool gt = cv > tv[q];
                      const float ov = tv[q];
                      const int32_t oi = ti[q];
                      tv[q] = gt ? cv : ov;
                      ti[q] = gt ? ci : oi;
                      cv = gt ? ov : cv;
                      ci = gt ? oi : ci;
                    }
                  }
                }
              }
            } else {
              const int d2 = (tile - p.vt_head) * 16 + vi;
              if (d2 < p.n_proj) p.out_proj[(int64_t)en * p.ld_proj + d2] = sum;
            }
          }
        }
        buf ^= 1;
      }
    }
  }

  if (p.out_head || p.vt_head == 0) return;

  // ---- merge the 16 residue lists of each row (16 consecutive lanes) into the workgroup's partial
  if (tid < 256) {
    const float mx = row16_max(run_m);
    const float s = row16_sum((run_m > SPEC_NEG_INF) ? run_s * __expf(run_m - mx) : 0.f);
    const int64_t slot = (int64_t)en * p.nparts + wg;
    if (en < R && vi == 0) {
      p.part.m[slot] = mx;
      p.part.s[slot] = s;
    }
    uint64_t hk[kMaxTopK];
#pragma unroll
    for (int q = 0; q < kMaxTopK; ++q) hk[q] = best_key(tv[q], ti[q]);
    const uint64_t kEmpty = best_key(SPEC_NEG_INF, kIdxNone);
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
      if (j < p.k_top) {
        const uint64_t best = row16_best_key(hk[0]);
        const bool won = hk[0] == best;   // the owner of the winner pops it
#pragma unroll
        for (int q = 0; q + 1 < kMaxTopK; ++q) {
          const uint64_t up = opaque_key(hk[q + 1]);
          hk[q] = won ? up : hk[q];
        }
        hk[kMaxTopK - 1] = won ? kEmpty : hk[kMaxTopK - 1];
        if (en < R && vi == j) {
          float bv;
          int32_t bi;
          best_unkey(best, bv, bi);
          p.part.val[slot * p.k_top + j] = bv;
          p.part.idx[slot * p.k_top + j] = bi;
        }
      }
    }
  }
}


}  // namespace specdraft
