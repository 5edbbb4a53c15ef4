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

#include <cstring>

#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

constexpr int KS = 2;   // K-steps (of 32) per slab
constexpr int PD = 3;   // slabs of global loads in flight ahead of the matrix cores
constexpr int NSET = PD + 1;

GemmPlan plan_gemm(int R, int n_rows_weight) {
  GemmPlan pl;
  if (R <= 32) { pl.mi = 2; pl.ni = 1; }
  else if (R <= 64) { pl.mi = 4; pl.ni = 1; }
  else { pl.mi = 8; pl.ni = 4; }
  pl.m_tiles = (R + 16 * pl.mi - 1) / (16 * pl.mi);
  pl.n_tiles = (n_rows_weight + 64 * pl.ni - 1) / (64 * pl.ni);
  return pl;
}

// Up to two weight matrices share one launch (head, then the next stage's
// projection): their workgroup tiles form one list, so the small projection
// fills the tail of the head's last wave of workgroups instead of a launch of its own.
struct GemmArgs {
  const u32x4* w[2];  // packed weights
  int nt_total[2];    // 16-row tiles of each weight matrix
  int n_valid[2];     // valid weight rows
  int n_tiles[2];     // workgroup tiles along the weight rows
  float* out[2];      // store epilogue target (matrix 0: only if mode0 == 1)
  int64_t ldo[2];
  int mode0;          // matrix 0: 0 = top-k partials, 1 = store.  Matrix 1 always stores.
  int kt;
  const u32x4* b;     // packed states
  int R, mt_total;
  int m_tiles, chunk; // chunk = workgroup tiles per XCD
  int k_top;
  Partials part;
  int nparts;
};

template <int MI, int NI>
__global__ __launch_bounds__(256) void head_gemm_kernel(GemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4* ldsB = reinterpret_cast<u32x4*>(smem);  // [2][MI*KS*64]
  constexpr int SLAB = MI * KS * 64;             // slots per slab
  constexpr int SPT = SLAB / 256;                // staging slots per thread
  static_assert(SLAB % 256 == 0, "a slab is staged by whole passes of the workgroup");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // XCD-aware tile id: hardware places workgroup ids round-robin over 8 XCDs
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  if (seq >= p.chunk) return;
  const int tile_id = xcd * p.chunk + seq;
  if (tile_id >= p.m_tiles * (p.n_tiles[0] + p.n_tiles[1])) return;
  int ntile = tile_id / p.m_tiles;
  const int mtile = tile_id - ntile * p.m_tiles;
  const int mat = ntile >= p.n_tiles[0] ? 1 : 0;
  ntile -= mat ? p.n_tiles[0] : 0;
  const int mode = mat ? 1 : p.mode0;
  const int n_valid = p.n_valid[mat];

  const int kt = p.kt;
  // weight fragments of this wave
  const u32x4* wptr[NI];
  int nt[NI];
#pragma unroll
  for (int ni = 0; ni < NI; ++ni) {
    nt[ni] = (ntile * 4 + wave) * NI + ni;
    const int ntc = min(nt[ni], p.nt_total[mat] - 1);
    wptr[ni] = p.w[mat] + (int64_t)ntc * kt * 64 + lane;
  }
  // staging sources of this thread
  const u32x4* sptr[SPT];
#pragma unroll
  for (int s = 0; s < SPT; ++s) {
    const int i = s * 256 + tid;
    const int mtl = i / (KS * 64), rem = i % (KS * 64);
    const int mt = min(mtile * MI + mtl, p.mt_total - 1);
    sptr[s] = p.b + (int64_t)mt * kt * 64 + rem;
  }

  f32x4 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Software pipeline over K-slabs.  Global loads (weight fragments into register
  // set a[], state slots into register set g[]) run PD slabs ahead; a state slab
  // is moved from its registers to LDS one slab before it is needed (LDS double
  // buffer, one barrier per slab).  NSET = PD + 1 register sets rotate through a
  // loop unrolled NSET times, so every index below is a compile-time constant.
  const int nslab = kt / KS;
  u32x4 a[NSET][NI][KS], g[NSET][SPT];
  auto load_slab = [&](u32x4 (&aw)[NI][KS], u32x4 (&gs)[SPT], int sl) {
    const int64_t off = (int64_t)sl * KS * 64;
#pragma unroll
    for (int s = 0; s < SPT; ++s) gs[s] = sptr[s][off];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int ts = 0; ts < KS; ++ts) aw[ni][ts] = wptr[ni][off + ts * 64];
  };
  auto store_s = [&](const u32x4 (&gs)[SPT], int buf) {
#pragma unroll
    for (int s = 0; s < SPT; ++s) ldsB[buf * SLAB + s * 256 + tid] = gs[s];
  };
  auto compute = [&](const u32x4 (&aw)[NI][KS], int buf) {
#pragma unroll
    for (int ts = 0; ts < KS; ++ts) {
      u32x4 bf[MI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) bf[mi] = ldsB[buf * SLAB + (mi * KS + ts) * 64 + lane];
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, aw[ni][ts]),
                                                                __builtin_bit_cast(bf16x8, bf[mi]), acc[mi][ni], 0, 0, 0);
    }
  };

#pragma unroll
  for (int q = 0; q < PD; ++q)
    if (q < nslab) load_slab(a[q], g[q], q);
  store_s(g[0], 0);
  __syncthreads();
  for (int base = 0; base < nslab; base += NSET) {
#pragma unroll
    for (int u = 0; u < NSET; ++u) {
      const int sl = base + u;
      if (sl < nslab) {
        if (sl + PD < nslab) load_slab(a[(u + PD) % NSET], g[(u + PD) % NSET], sl + PD);
        compute(a[u], u & 1);
        if (sl + 1 < nslab) store_s(g[(u + 1) % NSET], (u + 1) & 1);
        __syncthreads();
      }
    }
  }

  // ------------------------------------------------------------------ epilogue
  const int col = lane & 15, grp = lane >> 4;
  if (mode == 1) {
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int r = (mtile * MI + mi) * 16 + col;
      if (r >= p.R) continue;
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) {
        const int v0 = nt[ni] * 16 + grp * 4;
        float* o = p.out[mat] + (int64_t)r * p.ldo[mat] + v0;
        if (v0 + 3 < n_valid && (p.ldo[mat] & 3) == 0) {
          *reinterpret_cast<float4*>(o) = make_float4(acc[mi][ni][0], acc[mi][ni][1], acc[mi][ni][2], acc[mi][ni][3]);
        } else {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (v0 + i < n_valid) o[i] = acc[mi][ni][i];
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
        x[ni * 4 + i] = v < n_valid ? acc[mi][ni][i] : SPEC_NEG_INF;
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

hipError_t launch_head_gemm(const HeadJob& job, const GemmPlan& pl, hipStream_t st, hipEvent_t ev_start,
                            hipEvent_t ev_stop) {
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  int nm = 0;
  if (job.vt_head > 0) {
    a.w[nm] = static_cast<const u32x4*>(job.w_head);
    a.nt_total[nm] = job.vt_head;
    a.n_valid[nm] = job.n_head;
    a.n_tiles[nm] = (job.n_head + 64 * pl.ni - 1) / (64 * pl.ni);
    a.out[nm] = job.out_head;
    a.ldo[nm] = job.ld_head;
    a.mode0 = job.out_head ? 1 : 0;
    ++nm;
  }
  if (job.vt_proj > 0) {
    a.w[nm] = static_cast<const u32x4*>(job.w_proj);
    a.nt_total[nm] = job.vt_proj;
    a.n_valid[nm] = job.n_proj;
    a.n_tiles[nm] = (job.n_proj + 64 * pl.ni - 1) / (64 * pl.ni);
    a.out[nm] = job.out_proj;
    a.ldo[nm] = job.ld_proj;
    if (nm == 0) a.mode0 = 1;
    ++nm;
  }
  if (nm == 0) return hipErrorInvalidValue;
  a.kt = job.kt;
  a.b = static_cast<const u32x4*>(job.b_src);
  a.R = job.R;
  a.mt_total = (job.R + 15) / 16;
  a.m_tiles = pl.m_tiles;
  const int total = pl.m_tiles * (a.n_tiles[0] + a.n_tiles[1]);
  a.chunk = (total + 7) / 8;
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
