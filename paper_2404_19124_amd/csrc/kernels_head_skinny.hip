// Vocabulary head (and the next stage's projection) for at most 16 state rows:
// the bandwidth-bound batch-1 regime, where each stage streams its [V, D] head
// once against 1, k1, k1*k2 ... rows (Sec. 3.1 / 4.1 of the paper: 1, 6, 18 rows
// for the 6/3/2 tree).
//
// Design for CDNA4:
//  * one persistent workgroup of 16 waves per CU; tile = 16 weight rows x all of K;
//    workgroup g takes tiles g, g+G, g+2G ... of the combined list
//    [head tiles | next projection's tiles] (both consume the same states);
//  * K is split over the 16 waves; each wave streams its slice of the tile from
//    the tiled weight layout as fully coalesced 1 KiB fragments straight into
//    registers, DEPTH tiles ahead of the matrix-core work (a register ring of
//    DEPTH x NS fragments per wave: the loads of tile i+DEPTH are issued as the
//    registers of tile i are consumed);
//  * the states (<= 16 rows x K) sit in LDS for the whole kernel and feed the B
//    operand of v_mfma_f32_16x16x32_bf16; the A operand is the weight fragment,
//    so an accumulator lane holds 4 vocabulary entries of one state row;
//  * the 16 partial accumulators are summed through LDS (double-buffered, one
//    barrier per tile) by 256 threads, which keep per-thread running
//    (max, sum-exp, top-k) for "their" vocabulary residue; logits never leave
//    the CU.  At the end the workgroup writes one partial per row.
#include <hip/hip_ext.h>

#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

constexpr int kSkinnyWaves = 16;
constexpr int kSkinnySteps = 16;              // max K-steps (of 32) per wave -> K <= 8192
constexpr size_t kSkinnyLdsB = 128 * 1024;    // bytes available for the states
constexpr size_t kSkinnyLdsP = 2 * kSkinnyWaves * 64 * 16;  // partial accumulators, double-buffered

bool skinny_fits(int R, int kt) {
  if (R < 1 || R > 16) return false;
  if ((kt + kSkinnyWaves - 1) / kSkinnyWaves > kSkinnySteps) return false;
  return (size_t)R * kt * 4 * 16 <= kSkinnyLdsB;
}
int skinny_grid(int n_cu) { return n_cu > 0 ? n_cu : 256; }

// NS = K-steps per wave held per tile, DEPTH = tiles in flight per wave.
// EXACT: every wave has exactly NS steps (K = 16 * 32 * NS); otherwise waves
// take ceil(kt/16) <= NS steps with the tail predicated off.
template <int NS, int DEPTH, bool EXACT>
__global__ __launch_bounds__(kSkinnyWaves * 64) void head_skinny_kernel(HeadJob p) {
  extern __shared__ __align__(16) unsigned char smem[];
  const int kt = p.kt, R = p.R;
  u32x4* ldsB = reinterpret_cast<u32x4*>(smem);  // [kt][4][R] slots of 8 bf16
  const size_t bytesB = ((size_t)kt * 4 * R * 16 + 255) & ~(size_t)255;
  f32x4* ldsP = reinterpret_cast<f32x4*>(smem + bytesB);  // [2][waves][64]
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  constexpr int NT = kSkinnyWaves * 64;

  // ---- this wave's slice of K; the first tile's weights are requested before
  // anything else so that the stream is already in flight while the states load
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

  const int G = gridDim.x;
  u32x4 a[DEPTH][NS];
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {
    const int tile = blockIdx.x + d * G;
    if (tile < total) {
      const u32x4* ptr = tile_ptr(tile);
#pragma unroll
      for (int t = 0; t < NS; ++t)
        if (EXACT || t < ns) a[d][t] = ptr[t * 64];
    }
  }

  // ---- states -> LDS, trimmed to R rows: slot (t, g, n) = row n, columns t*32 + g*8 .. +8
  for (int slot = tid; slot < kt * 4 * R; slot += NT) {
    const int n = slot % R, tg = slot / R;
    u32x4 v;
    if (p.b_rowmajor)
      v = *reinterpret_cast<const u32x4*>(static_cast<const uint16_t*>(p.b_src) + (int64_t)n * p.b_ld + tg * 8);
    else
      v = static_cast<const u32x4*>(p.b_src)[(int64_t)(tg >> 2) * 64 + (tg & 3) * 16 + n];
    ldsB[slot] = v;
  }
  __syncthreads();

  // running state of the 256 epilogue threads: state row en, vocabulary residue vi
  const int en = tid & 15, vi = (tid >> 4) & 15;
  float run_m = SPEC_NEG_INF, run_s = 0.f;
  float tv[kMaxTopK];
  int32_t ti[kMaxTopK];
#pragma unroll
  for (int q = 0; q < kMaxTopK; ++q) { tv[q] = SPEC_NEG_INF; ti[q] = kIdxNone; }

  int buf = 0;
  for (int base = blockIdx.x; base < total; base += DEPTH * G) {
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
            if (has_next) a[d][t] = nptr[t * 64];
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

  // ---- merge the 16 residue lists of each row into the workgroup's partial
  __syncthreads();
  float* lv = reinterpret_cast<float*>(ldsP);               // [16 rows][16 vi][8]
  int32_t* li = reinterpret_cast<int32_t*>(lv + 16 * 16 * kMaxTopK);
  float* lm = reinterpret_cast<float*>(li + 16 * 16 * kMaxTopK);  // [16][16]
  float* ls = lm + 256;
  if (tid < 256) {
#pragma unroll
    for (int q = 0; q < kMaxTopK; ++q) {
      lv[(en * 16 + vi) * kMaxTopK + q] = tv[q];
      li[(en * 16 + vi) * kMaxTopK + q] = ti[q];
    }
    lm[en * 16 + vi] = run_m;
    ls[en * 16 + vi] = run_s;
  }
  __syncthreads();
  if (tid < 256) {
    // now 16 consecutive lanes own one row: row = tid/16, list = tid%16
    const int row = tid >> 4, src = tid & 15;
    float hv[kMaxTopK];
    int32_t hi[kMaxTopK];
#pragma unroll
    for (int q = 0; q < kMaxTopK; ++q) {
      hv[q] = lv[(row * 16 + src) * kMaxTopK + q];
      hi[q] = li[(row * 16 + src) * kMaxTopK + q];
    }
    float m = lm[row * 16 + src], s = ls[row * 16 + src];
    const float mx = row16_max(m);
    s = row16_sum((m > SPEC_NEG_INF) ? s * __expf(m - mx) : 0.f);
    const int64_t slot = (int64_t)row * p.nparts + blockIdx.x;
    if (row < R && src == 0) {
      p.part.m[slot] = mx;
      p.part.s[slot] = s;
    }
#pragma unroll
    for (int j = 0; j < kMaxTopK; ++j) {
      if (j < p.k_top) {
        float bv = hv[0];
        int32_t bi = hi[0];
        row16_best(bv, bi);
        if (hi[0] == bi && hv[0] == bv) {  // the owner of the winner pops it
#pragma unroll
          for (int q = 0; q + 1 < kMaxTopK; ++q) { hv[q] = hv[q + 1]; hi[q] = hi[q + 1]; }
          hv[kMaxTopK - 1] = SPEC_NEG_INF;
          hi[kMaxTopK - 1] = kIdxNone;
        }
        if (row < R && src == j) {
          p.part.val[slot * p.k_top + j] = bv;
          p.part.idx[slot * p.k_top + j] = bi;
        }
      }
    }
  }
}

template <int NS, int DEPTH, bool EXACT>
static hipError_t launch_skinny_t(const HeadJob& job, int grid, size_t smem, hipStream_t st, hipEvent_t ev_start,
                                  hipEvent_t ev_stop) {
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(head_skinny_kernel<NS, DEPTH, EXACT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kSkinnyLdsB + kSkinnyLdsP));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipExtLaunchKernelGGL((head_skinny_kernel<NS, DEPTH, EXACT>), dim3(grid), dim3(kSkinnyWaves * 64), smem, st,
                        ev_start, ev_stop, 0, job);
  return hipGetLastError();
}

hipError_t launch_head_skinny(const HeadJob& job, int n_cu, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const size_t bytesB = ((size_t)job.kt * 4 * job.R * 16 + 255) & ~(size_t)255;
  const size_t smem = bytesB + kSkinnyLdsP;
  const int grid = skinny_grid(n_cu);
  // K = 512 * NS gets an exact instantiation with as many tiles in flight as 16 fragments allow
  switch (job.kt % kSkinnyWaves == 0 ? job.kt / kSkinnyWaves : 0) {
    case 4: return launch_skinny_t<4, 4, true>(job, grid, smem, st, ev_start, ev_stop);
    case 6: return launch_skinny_t<6, 2, true>(job, grid, smem, st, ev_start, ev_stop);
    case 8: return launch_skinny_t<8, 2, true>(job, grid, smem, st, ev_start, ev_stop);
    case 10: return launch_skinny_t<10, 1, true>(job, grid, smem, st, ev_start, ev_stop);
    case 16: return launch_skinny_t<16, 1, true>(job, grid, smem, st, ev_start, ev_stop);
    default: return launch_skinny_t<kSkinnySteps, 1, false>(job, grid, smem, st, ev_start, ev_stop);
  }
}

}  // namespace specdraft
