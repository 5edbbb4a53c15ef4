// Vocabulary head / state projection as a dense bf16 contraction on the matrix
// cores, for any number of state rows (the batch >= 2 regime: 64, 320, 960 rows
// per stage for 64 sequences with a 5/3/2 tree).
//
// Design for CDNA4:
//  * workgroup = 4 waves; workgroup tile = (16*MI state rows) x (4 * NI * 16
//    weight rows); every wave owns NI*16 weight rows and all 16*MI state rows,
//    so no weight fragment is loaded twice inside a workgroup;
//  * weights come from the tiled layout as coalesced 1 KiB fragments straight
//    into registers (A operand of v_mfma_f32_16x16x32_bf16), prefetched one
//    K-slab ahead; states (B operand) are staged through LDS, double-buffered,
//    one barrier per slab.  The states are already stored in fragment order, so
//    the global->LDS copy is linear and the LDS reads are conflict-free;
//  * accumulator lane l holds state row l%16 and 4 weight rows: the softmax /
//    top-k reduction over the vocabulary is mostly lane-local.  The epilogue
//    keeps, per (row, workgroup tile), max, sum-exp and the k best logits;
//    logits are never written to memory (unless the store epilogue is asked for);
//  * workgroup ids are remapped so that the tiles of one XCD (ids congruent
//    mod 8) walk a contiguous range of weight-row tiles with the state-row tile
//    varying fastest: workgroups that share weights run together on one L2.
#include <hip/hip_ext.h>

#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

constexpr int KS = 2;  // K-steps (of 32) per slab

GemmPlan plan_gemm(int R, int n_rows_weight) {
  GemmPlan pl;
  if (R <= 32) { pl.mi = 2; pl.ni = 1; }
  else if (R <= 64) { pl.mi = 4; pl.ni = 1; }
  else { pl.mi = 8; pl.ni = 4; }
  pl.m_tiles = (R + 16 * pl.mi - 1) / (16 * pl.mi);
  pl.n_tiles = (n_rows_weight + 64 * pl.ni - 1) / (64 * pl.ni);
  return pl;
}

struct GemmArgs {
  const uint4* w;     // packed weights
  int nt_total;       // 16-row tiles of the weight matrix
  int n_valid;        // valid weight rows
  int kt;
  const uint4* b;     // packed states
  int R, mt_total;
  int m_tiles, n_tiles, chunk;  // chunk = workgroup tiles per XCD
  int mode;           // 0: top-k partials, 1: store
  int k_top;
  Partials part;
  int nparts;
  float* out;
  int64_t ldo;
};

template <int MI, int NI>
__global__ __launch_bounds__(256) void head_gemm_kernel(GemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem[];
  uint4* ldsB = reinterpret_cast<uint4*>(smem);  // [2][MI*KS*64]
  constexpr int SLAB = MI * KS * 64;             // slots per slab
  constexpr int SPT = (SLAB + 255) / 256;        // staging slots per thread
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // XCD-aware tile id: hardware places workgroup ids round-robin over 8 XCDs
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  if (seq >= p.chunk) return;
  const int tile_id = xcd * p.chunk + seq;
  if (tile_id >= p.m_tiles * p.n_tiles) return;
  const int ntile = tile_id / p.m_tiles, mtile = tile_id - ntile * p.m_tiles;

  const int kt = p.kt;
  // weight fragments of this wave
  const uint4* wptr[NI];
  int nt[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    nt[ni] = (ntile * 4 + wave) * NI + ni;
    const int ntc = min(nt[ni], p.nt_total - 1);
    wptr[ni] = p.w + (int64_t)ntc * kt * 64 + lane;
  }
  // staging sources of this thread
  const uint4* sptr[SPT];
#pragma unroll
  for (int s = 0; s < SPT; ++s) {
    const int i = s * 256 + tid;
    const int mtl = min(i / (KS * 64), MI - 1), rem = i % (KS * 64);
    const int mt = min(mtile * MI + mtl, p.mt_total - 1);
    sptr[s] = p.b + (int64_t)mt * kt * 64 + rem;
  }

  f32x4 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const int nslab = kt / KS;
  uint4 a_cur[NI][KS], a_nxt[NI][KS], stg[SPT];
  // prologue: slab 0
#pragma unroll
  for (int s = 0; s < SPT; ++s)
    if (s * 256 + tid < SLAB) stg[s] = sptr[s][0];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni)
#pragma unroll
    for (int ts = 0; ts < KS; ++ts) a_cur[ni][ts] = wptr[ni][ts * 64];
#pragma unroll
  for (int s = 0; s < SPT; ++s)
    if (s * 256 + tid < SLAB) ldsB[s * 256 + tid] = stg[s];
  __syncthreads();

  for (int sl = 0; sl < nslab; ++sl) {
    const int cur = sl & 1;
    const bool more = sl + 1 < nslab;
    if (more) {
      const int64_t off = (int64_t)(sl + 1) * KS * 64;
#pragma unroll
      for (int s = 0; s < SPT; ++s)
        if (s * 256 + tid < SLAB) stg[s] = sptr[s][off];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int ts = 0; ts < KS; ++ts) a_nxt[ni][ts] = wptr[ni][off + ts * 64];
    }
#pragma unroll
    for (int ts = 0; ts < KS; ++ts) {
      uint4 bf[MI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) bf[mi] = ldsB[cur * SLAB + (mi * KS + ts) * 64 + lane];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a_cur[ni][ts]),
                                                                __builtin_bit_cast(bf16x8, bf[mi]), acc[mi][ni], 0, 0, 0);
    }
    if (more) {
#pragma unroll
      for (int s = 0; s < SPT; ++s)
        if (s * 256 + tid < SLAB) ldsB[(cur ^ 1) * SLAB + s * 256 + tid] = stg[s];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int ts = 0; ts < KS; ++ts) a_cur[ni][ts] = a_nxt[ni][ts];
    }
    __syncthreads();
  }

  // ------------------------------------------------------------------ epilogue
  const int col = lane & 15, grp = lane >> 4;
  if (p.mode == 1) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int r = (mtile * MI + mi) * 16 + col;
      if (r >= p.R) continue;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int v0 = nt[ni] * 16 + grp * 4;
        float* o = p.out + (int64_t)r * p.ldo + v0;
        if (v0 + 3 < p.n_valid && (p.ldo & 3) == 0) {
          *reinterpret_cast<float4*>(o) = make_float4(acc[mi][ni][0], acc[mi][ni][1], acc[mi][ni][2], acc[mi][ni][3]);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (v0 + i < p.n_valid) o[i] = acc[mi][ni][i];
        }
      }
    }
    return;
  }

  // top-k partials.  LDS scratch (aliases the slabs; the main loop ended on a barrier):
  //   sv/si [4 waves][16*MI rows][k_top], sm/ss [4][16*MI]
  const int k_top = p.k_top;
  constexpr int ROWS = 16 * MI;
  float* sv = reinterpret_cast<float*>(smem);
  int32_t* si = reinterpret_cast<int32_t*>(sv + 4 * ROWS * kMaxTopK);
  float* sm = reinterpret_cast<float*>(si + 4 * ROWS * kMaxTopK);
  float* ss = sm + 4 * ROWS;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    // this lane's 4*NI logits of state row (mi, col), in increasing vocabulary order
    float x[NI * 4];
    int32_t vx[NI * 4];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int v = nt[ni] * 16 + grp * 4 + i;
        vx[ni * 4 + i] = v;
        x[ni * 4 + i] = v < p.n_valid ? acc[mi][ni][i] : SPEC_NEG_INF;
      }
    float lastv = __builtin_huge_valf();
    int32_t lasti = -1;
    float mx = SPEC_NEG_INF;
    const int rl = mi * 16 + col;
    for (int j = 0; j < k_top; ++j) {
      float bv = SPEC_NEG_INF;
      int32_t bi = kIdxNone;
#pragma unroll
      for (int e = 0; e < NI * 4; ++e)
        if (before(lastv, lasti, x[e], vx[e]) && before(x[e], vx[e], bv, bi)) { bv = x[e]; bi = vx[e]; }
#pragma unroll
      for (int o = 32; o >= 16; o >>= 1) {
        const float ov = __shfl_xor(bv, o, 64);
        const int32_t oi = __shfl_xor(bi, o, 64);
        if (before(ov, oi, bv, bi)) { bv = ov; bi = oi; }
      }
      if (j == 0) mx = bv;
      if (grp == 0) {
        sv[(wave * ROWS + rl) * kMaxTopK + j] = bv;
        si[(wave * ROWS + rl) * kMaxTopK + j] = bi;
      }
      lastv = bv;
      lasti = bi;
    }
    float s = 0.f;
    if (mx > SPEC_NEG_INF) {
#pragma unroll
      for (int e = 0; e < NI * 4; ++e) s += __expf(x[e] - mx);
    }
    s += __shfl_xor(s, 16, 64);
    s += __shfl_xor(s, 32, 64);
    if (grp == 0) {
      sm[wave * ROWS + rl] = mx;
      ss[wave * ROWS + rl] = s;
    }
  }
  __syncthreads();
  if (tid < ROWS) {
    const int r = mtile * ROWS + tid;
    if (r < p.R) {
      float mx = sm[tid];
#pragma unroll
      for (int w = 1; w < 4; ++w) mx = fmaxf(mx, sm[w * ROWS + tid]);
      float s = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float m = sm[w * ROWS + tid];
        if (m > SPEC_NEG_INF) s += ss[w * ROWS + tid] * __expf(m - mx);
      }
      const int64_t slot = (int64_t)r * p.nparts + ntile;
      p.part.m[slot] = mx;
      p.part.s[slot] = s;
      int ptr[4] = {0, 0, 0, 0};
      for (int j = 0; j < k_top; ++j) {
        float bv = SPEC_NEG_INF;
        int32_t bi = kIdxNone;
        int bw = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          if (ptr[w] < k_top) {
            const float v = sv[(w * ROWS + tid) * kMaxTopK + ptr[w]];
            const int32_t i = si[(w * ROWS + tid) * kMaxTopK + ptr[w]];
            if (before(v, i, bv, bi)) { bv = v; bi = i; bw = w; }
          }
        }
#pragma unroll
        for (int w = 0; w < 4; ++w)
          if (w == bw) ptr[w]++;
        p.part.val[slot * k_top + j] = bv;
        p.part.idx[slot * k_top + j] = bi;
      }
    }
  }
}

static size_t gemm_smem(int mi) {
  const size_t slabs = (size_t)2 * mi * KS * 64 * 16;
  const size_t rows = 16 * (size_t)mi;
  const size_t epi = 4 * rows * kMaxTopK * 8 + 4 * rows * 8;
  return slabs > epi ? slabs : epi;
}

hipError_t launch_head_gemm(const HeadJob& job, bool proj_matrix, const GemmPlan& pl, hipStream_t st,
                            hipEvent_t ev_start, hipEvent_t ev_stop) {
  GemmArgs a;
  a.w = static_cast<const uint4*>(proj_matrix ? job.w_proj : job.w_head);
  a.nt_total = proj_matrix ? job.vt_proj : job.vt_head;
  a.n_valid = proj_matrix ? job.n_proj : job.n_head;
  a.kt = job.kt;
  a.b = static_cast<const uint4*>(job.b_src);
  a.R = job.R;
  a.mt_total = (job.R + 15) / 16;
  a.m_tiles = pl.m_tiles;
  a.n_tiles = pl.n_tiles;
  const int total = pl.m_tiles * pl.n_tiles;
  a.chunk = (total + 7) / 8;
  if (proj_matrix) {
    a.mode = 1;
    a.out = job.out_proj;
    a.ldo = job.ld_proj;
  } else if (job.out_head) {
    a.mode = 1;
    a.out = job.out_head;
    a.ldo = job.ld_head;
  } else {
    a.mode = 0;
    a.out = nullptr;
    a.ldo = 0;
  }
  a.k_top = job.k_top;
  a.part = job.part;
  a.nparts = job.nparts;
  dim3 grid(a.chunk * 8), block(256);
  const size_t smem = gemm_smem(pl.mi);
  if (pl.mi == 2 && pl.ni == 1) hipExtLaunchKernelGGL((head_gemm_kernel<2, 1>), grid, block, smem, st, ev_start, ev_stop, 0, a);
  else if (pl.mi == 4 && pl.ni == 1) hipExtLaunchKernelGGL((head_gemm_kernel<4, 1>), grid, block, smem, st, ev_start, ev_stop, 0, a);
  else if (pl.mi == 8 && pl.ni == 4) hipExtLaunchKernelGGL((head_gemm_kernel<8, 4>), grid, block, smem, st, ev_start, ev_stop, 0, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace specdraft
