// Vocabulary head / state projection as a dense bf16 contraction on the matrix
// cores, for any number of state rows (the batch >= 2 regime: 64, 320, 960 rows
// per stage for 64 sequences with a 5/3/2 tree).
//
// Design for CDNA4:
//  * workgroup = 4 waves, one per SIMD; workgroup tile = (16*MI state rows) x
//    (4 * NI * 16 weight rows); every wave owns NI*16 weight rows and all 16*MI
//    state rows, so no weight fragment is loaded twice inside a workgroup;
//  * weights come from the tiled layout as coalesced 1 KiB fragments straight
//    into registers (A operand of v_mfma_f32_16x16x32_bf16); states (B operand)
//    are staged through LDS (they are stored in fragment order already, so the
//    copy is linear and the reads are conflict-free).  Global loads run PD
//    K-slabs ahead of the matrix cores through rotating register sets;
//  * a workgroup is persistent over a contiguous RANGE of weight-row tiles for
//    its block of state rows.  That is what makes the fused epilogue cheap: every
//    lane carries, per state row, a running (max, sum-exp) and a short sorted
//    top-k list across the tiles of its range, so a new logit costs one exp and
//    one compare against the lane's current k-th best (insertions become rare
//    after the first tile).  Logits are never written to memory.  The lists of
//    the 16 lanes that share a row are merged once, when the range is done;
//  * the next stage's projection rides in the same launch: its tiles follow the
//    head's in the tile list (store epilogue);
//  * workgroup ids are remapped so that the workgroups of one XCD (ids congruent
//    mod 8) share ranges with the state-row block varying fastest: workgroups
//    that stream the same weights run together on one L2.
#include <hip/hip_ext.h>

#include <cstring>

#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

// Slab geometry: KS K-steps (of 32) per slab; weight loads run PD slabs ahead of the
// matrix cores through NSET = PD + 1 rotating register sets; a state slab is written to
// one of NSET LDS buffers TWO slabs before it is used, so that the fragments of the next
// slab's first K-step can be read before the barrier that closes the current slab and the
// matrix cores never wait for LDS behind a barrier.
constexpr int KS = 2;
constexpr int PD = 3;
constexpr int NSET = PD + 1;
// State slots are requested GD slabs ahead of their USE, i.e. GD - 2 slabs ahead of the
// copy into LDS (which happens two slabs before the use): with GD = PD the copy would
// wait for loads issued just one slab earlier, and, loads completing in order, for
// everything issued before them.
constexpr int GD = 4;
static_assert(GD <= NSET, "a state register set is reused NSET slabs later");

// Cost of one tile with 128- / 160-row state blocks relative to one with 96-row blocks
// (measured at the 7B shape: 54, 65 and 76 us per tile of a range).
constexpr double kMidSlabCost = 1.2;
constexpr double kTallSlabCost = 1.4;

// Workgroup tiles of the two weight matrices for tiles of ts 16-row weight tiles.
static int plan_tiles(int n_rows, int ts) { return ((n_rows + 15) / 16 + ts - 1) / ts; }

static void fill_plan(GemmPlan& pl, int R, int n_head, int n_proj, int n_cu) {
  pl.m_tiles = (R + 16 * pl.mi - 1) / (16 * pl.mi);
  const int nt_head = plan_tiles(n_head, pl.ts);
  const int nt_proj = plan_tiles(n_proj, pl.ts);
  const int total = nt_head + nt_proj;
  // narrow blocks are bandwidth-bound and light on registers: two workgroups per CU keep more loads in flight
  int nr = (pl.ni == 1 ? 2 : 1) * (n_cu > 0 ? n_cu : 256) / pl.m_tiles;
  if (nr < 1) nr = 1;
  if (nr > total) nr = total;
  pl.n_ranges = nr;
  // ranges are the balanced split t0(r) = r * total / nr; those that start inside the head hold head tiles
  int np = 0;
  while (np < nr && (int64_t)np * total / nr < nt_head) ++np;
  pl.nparts = np;
}

// Wide kernel with at most one 256-row tile per range (fewer tiles than CUs: an HBM-bound
// launch that leaves CUs idle): the smallest tile, in 16-row weight tiles, that still gives every
// range at most one.  A tile costs its K loop whether all four waves have valid rows or not, but
// every range then streams fewer weight rows and the idle ranges get one: 157 tiles of 256 rows
// over 256 CUs become 252 tiles of 160.  (With several tiles per range the launch is bound by
// the matrix cores or the L2, and more K loops only cost: measured.)
static void shrink_tile(GemmPlan& pl, int R, int n_head, int n_proj, int n_cu) {
  const int per16 = (plan_tiles(n_head, 16) + plan_tiles(n_proj, 16) + pl.n_ranges - 1) / pl.n_ranges;
  if (per16 > 1) return;
  for (int ts = 4; ts < 16; ++ts) {
    GemmPlan c = pl;
    c.ts = ts;
    fill_plan(c, R, n_head, n_proj, n_cu);
    const int per = (plan_tiles(n_head, ts) + plan_tiles(n_proj, ts) + c.n_ranges - 1) / c.n_ranges;
    if (per <= per16) { pl = c; return; }
  }
}

GemmPlan plan_gemm(int R, int k_top, int n_head, int n_proj, int kt, int n_cu) {
  GemmPlan pl;
  pl.ts = 4;
  pl.ksplit = 1;
  if (R <= 32) { pl.mi = 2; pl.ni = 1; pl.kcap = 8; }
  // 33..64 rows against a long weight matrix (at least one 256-row tile per two CUs): the
  // wide kernel re-reads the states a quarter as often per weight byte as the narrow one
  else if (R <= 64 && (int64_t)n_head + n_proj >= (int64_t)128 * (n_cu > 0 ? n_cu : 256)) {
    pl.mi = 4; pl.ni = 4; pl.ts = 16;
    pl.kcap = k_top <= 2 ? 2 : (k_top <= 4 ? 4 : (k_top <= 6 ? 6 : 8));
    fill_plan(pl, R, n_head, n_proj, n_cu);
    shrink_tile(pl, R, n_head, n_proj, n_cu);
    return pl;
  }
  else if (R <= 64) {
    // a short weight matrix (a projection alone) has too few 64-row tiles to fill the chip with
    // 64-row state blocks: two 32-row blocks double the workgroups (the second reads the weights from L2)
    const int64_t tiles = ((int64_t)n_head + 63) / 64 + ((int64_t)n_proj + 63) / 64;
    pl.mi = tiles < (n_cu > 0 ? n_cu : 256) ? 2 : 4;
    pl.ni = 1;
    pl.kcap = 8;
  }
  else {
    // wide kernel; the per-lane top-k lists are as short as k_top allows (the epilogue of a tile is the
    // insertion of every logit into them: its cost grows with their length, and a single-tile launch
    // ends on it)
    pl.ni = 4;
    pl.ts = 16;
    pl.kcap = k_top <= 4 ? (k_top < 2 ? 2 : k_top) : (k_top <= 6 ? 6 : 8);
    pl.mi = 6;
    fill_plan(pl, R, n_head, n_proj, n_cu);
    if (pl.kcap <= 4) {
      // 96-, 128- or 160-row state blocks: the longest range decides the launch; a tile of a
      // taller block costs more (measured per K slab, relative to the 96-row block), but less
      // than its share of rows (more matrix work per byte from L2)
      const int total = (n_head + 255) / 256 + (n_proj + 255) / 256;
      double best = 1.0 * ((total + pl.n_ranges - 1) / pl.n_ranges);
      const int cand_mi[2] = {8, 10};
      const double cand_cost[2] = {kMidSlabCost, kTallSlabCost};
      for (int c = 0; c < 2; ++c) {
        GemmPlan alt = pl;
        alt.mi = cand_mi[c];
        fill_plan(alt, R, n_head, n_proj, n_cu);
        const double cost = cand_cost[c] * ((total + alt.n_ranges - 1) / alt.n_ranges);
        if (cost < best) { best = cost; pl = alt; }
      }
    }
    // a projection alone: a few dozen workgroups; K is split over more (all four waves stay busy, which
    // short tiles would not give; the consumer adds the parts)
    if (n_head == 0) {
      const int cus = n_cu > 0 ? n_cu : 256;
      while (pl.ksplit < kMaxKSplit && pl.m_tiles * pl.n_ranges * pl.ksplit * 2 <= cus && kt / KS / (pl.ksplit * 2) >= 8)
        pl.ksplit *= 2;
    }
    if (pl.ksplit == 1) shrink_tile(pl, R, n_head, n_proj, n_cu);
    return pl;
  }
  fill_plan(pl, R, n_head, n_proj, n_cu);
  // A projection alone is a short weight matrix: a few dozen workgroups, each with a long
  // serial K loop and only its own prefetch depth in flight.  Splitting K over more
  // workgroups multiplies the bytes in flight; the consumer adds the partial sums.
  if (n_head == 0) {
    const int cus = n_cu > 0 ? n_cu : 256;
    while (pl.ksplit < kMaxKSplit && pl.m_tiles * pl.n_ranges * pl.ksplit * 2 <= 2 * cus &&
           kt / KS / (pl.ksplit * 2) >= 8)
      pl.ksplit *= 2;
  }
  return pl;
}

// Cost of a launch in units of one 96-row-block tile: the longest range decides.
static double plan_cost(const GemmPlan& pl, int n_head, int n_proj) {
  const int total = plan_tiles(n_head, pl.ts) + plan_tiles(n_proj, pl.ts);
  const double per_tile = pl.mi >= 10 ? kTallSlabCost : (pl.mi >= 8 ? kMidSlabCost : 1.0);
  return per_tile * ((total + pl.n_ranges - 1) / pl.n_ranges) / pl.ksplit;
}

// Head and next projection in ONE launch share the state reads, but their tiles form one list, and a list
// that is a little longer than a multiple of the ranges makes the launch one tile longer for a few ranges
// (320 rows against 125 + 16 tiles: 128 ranges, 13 of them with two tiles).  Then two launches are cheaper:
// the head alone in one even round, the projection alone split along K over the whole chip.
bool plan_projection_apart(int R, int k_top, int n_head, int n_proj, int kt, int n_cu) {
  if (R <= 64 || n_head <= 0 || n_proj <= 0) return false;   // wide kernel only
  const GemmPlan both = plan_gemm(R, k_top, n_head, n_proj, kt, n_cu);
  const GemmPlan head = plan_gemm(R, k_top, n_head, 0, kt, n_cu);
  const GemmPlan proj = plan_gemm(R, 0, 0, n_proj, kt, n_cu);
  if (both.ni != 4 || head.ni != 4 || proj.ni != 4) return false;
  const double launch = 0.15;   // a second launch: drain, start, pipeline fill, partial sums read back
  return plan_cost(head, n_head, 0) + plan_cost(proj, 0, n_proj) + launch < plan_cost(both, n_head, n_proj) - 0.05;
}

struct GemmArgs {
  const u32x4* w[2];  // packed weights: matrix 0 = head (or the only matrix), 1 = projection
  int nt_total[2];    // 16-row tiles of each weight matrix
  int n_valid[2];     // valid weight rows
  int n_tiles[2];     // workgroup tiles along the weight rows
  float* out[2];      // store epilogue target
  int64_t ldo[2];
  int mode0;          // matrix 0: 0 = top-k partials, 1 = store.  Matrix 1 always stores.
  int kt;
  const u32x4* b;     // states: packed tiles, or (narrow kernel only) row-major bf16 [R][b_ld] if b_rowmajor
  int b_rowmajor, b_ld;
  int R, mt_total;
  int m_tiles, n_ranges, chunk;  // chunk = workgroups per XCD
  int ts;                        // 16-row weight tiles per workgroup tile (wide kernel)
  int ksplit;                    // a projection alone (store epilogue): workgroups per tile along K
  int64_t out_part_stride;       // floats between the K parts' outputs
  int k_top;
  Partials part;
  int nparts;
};

// Narrow blocks (MI <= 4) are bandwidth-bound: two workgroups per CU (two waves per
// SIMD, 256 registers each) keep twice the loads in flight; wide blocks take all 512.
template <int MI, int NI, int KT>
__global__ __launch_bounds__(256, (MI <= 4 ? 2 : 1)) void head_gemm_kernel(GemmArgs p) {
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4* ldsB = reinterpret_cast<u32x4*>(smem);  // [NSET][MI*KS*64]
  constexpr int SLAB = MI * KS * 64;             // slots per slab
  constexpr int SPT = SLAB / 256;                // staging slots per thread
  static_assert(SLAB % 256 == 0, "a slab is staged by whole passes of the workgroup");
  static_assert(KS == 2, "the K loop below is written for two K-steps per slab");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int col = lane & 15, grp = lane >> 4;

  // XCD-aware workgroup id: hardware places workgroup ids round-robin over 8 XCDs
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  if (seq >= p.chunk) return;
  const int wg = xcd * p.chunk + seq;
  if (wg >= p.m_tiles * p.n_ranges * p.ksplit) return;
  // K split (store epilogue only): part kpart of a tile covers slabs [slab0, slab0 + nslab)
  const int kpart = wg % p.ksplit, wg2 = wg / p.ksplit;
  const int range = wg2 / p.m_tiles, mtile = wg2 - range * p.m_tiles;
  const int total_tiles = p.n_tiles[0] + p.n_tiles[1];
  const int t0 = (int)((int64_t)range * total_tiles / p.n_ranges);
  const int t1 = (int)((int64_t)(range + 1) * total_tiles / p.n_ranges);

  const int kt = p.kt;
  const int slab0 = (int)((int64_t)kpart * (kt / KS) / p.ksplit);
  const int nslab = (int)((int64_t)(kpart + 1) * (kt / KS) / p.ksplit) - slab0;
  // staging sources of this thread (the same for every tile of the range)
  const u32x4* sptr[SPT];
#pragma unroll
  for (int s = 0; s < SPT; ++s) {
    const int i = s * 256 + tid;
    const int mtl = i / (KS * 64), rem = i % (KS * 64);
    const int mt = min(mtile * MI + mtl, p.mt_total - 1);
    if (p.b_rowmajor) {
      // gather the slot from the caller's row-major rows: slot (K step ts, lane l) of a 16-row tile holds
      // row l % 16, columns 32 ts + 8 (l / 16) .. + 8; a slab further on is KS * 32 columns = KS * 4 slots
      const int ts = rem >> 6, l = rem & 63;
      const int row = min(mt * 16 + (l & 15), p.R - 1);   // rows past R are masked in the epilogue
      sptr[s] = p.b + ((int64_t)row * p.b_ld + ((int64_t)slab0 * KS + ts) * 32 + (l >> 4) * 8) / 8;
    } else {
      sptr[s] = p.b + (int64_t)mt * kt * 64 + (int64_t)slab0 * KS * 64 + rem;
    }
  }

  // weight fragment pointers of this wave for a given tile of the list
  const u32x4* wptr[NI];
  auto set_tile = [&](int t, const u32x4* (&wp)[NI], int (&ntv)[NI], int& mat) {
    mat = t >= p.n_tiles[0] ? 1 : 0;
    const int ntile = t - (mat ? p.n_tiles[0] : 0);
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
      ntv[ni] = (ntile * 4 + wave) * NI + ni;
      const int ntc = min(ntv[ni], p.nt_total[mat] - 1);
      wp[ni] = p.w[mat] + (int64_t)ntc * kt * 64 + (int64_t)slab0 * KS * 64 + lane;
    }
  };

  // Rotating register sets: weight fragments a[], state slots g[].
  u32x4 a[NSET][NI][KS], g[NSET][SPT];
  auto load_g = [&](u32x4 (&gs)[SPT], int sl) {
    const int64_t off = (int64_t)sl * KS * (p.b_rowmajor ? 4 : 64);
#pragma unroll
    for (int s = 0; s < SPT; ++s) gs[s] = sptr[s][off];
  };
  auto load_a = [&](u32x4 (&aw)[NI][KS], int sl) {
    const int64_t off = (int64_t)sl * KS * 64;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int ts = 0; ts < KS; ++ts) aw[ni][ts] = wptr[ni][off + ts * 64];
  };
  auto store_s = [&](const u32x4 (&gs)[SPT], int buf) {
#pragma unroll
    for (int s = 0; s < SPT; ++s) ldsB[buf * SLAB + s * 256 + tid] = gs[s];
  };

  // running softmax / top-k state of this lane, per state row (mi, col)
  float run_m[MI], run_s[MI], lv[MI][KT];
  int32_t li[MI][KT];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    run_m[mi] = SPEC_NEG_INF;
    run_s[mi] = 0.f;
#pragma unroll
    for (int q = 0; q < KT; ++q) { lv[mi][q] = SPEC_NEG_INF; li[mi][q] = kIdxNone; }
  }
  bool any_head = false;

  int nt[NI], mat = 0;
  set_tile(t0, wptr, nt, mat);
#pragma unroll
  for (int q = 0; q < GD; ++q)
    if (q < nslab) load_g(g[q], q);
#pragma unroll
  for (int q = 0; q < PD; ++q)
    if (q < nslab) load_a(a[q], q);

  for (int t = t0; t < t1; ++t) {
    f32x4 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
      for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = (f32x4){0.f, 0.f, 0.f, 0.f};
    auto read_b = [&](u32x4 (&bf)[MI], int buf, int ts) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) bf[mi] = ldsB[buf * SLAB + (mi * KS + ts) * 64 + lane];
    };
    auto mma = [&](const u32x4 (&aw)[NI][KS], const u32x4 (&bf)[MI], int ts) {
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, aw[ni][ts]),
                                                                __builtin_bit_cast(bf16x8, bf[mi]), acc[mi][ni], 0, 0, 0);
    };

    // ---- K loop (slab sl uses register set and LDS buffer sl % NSET; the loop is
    // unrolled NSET times so every index is a constant)
    store_s(g[0], 0);
    if (nslab > 1) store_s(g[1], 1);
    __syncthreads();
    u32x4 bf0[MI], bf1[MI];
    read_b(bf0, 0, 0);
    int base = 0;
    // steady state: no branches inside, so the compiler's wait counters see
    // straight-line code and let all PD slabs of loads stay in flight
    for (; base + NSET + GD <= nslab; base += NSET) {
#pragma unroll
      for (int u = 0; u < NSET; ++u) {
        load_g(g[(u + GD) % NSET], base + u + GD);
        load_a(a[(u + PD) % NSET], base + u + PD);
        read_b(bf1, u, 1);
        mma(a[u], bf0, 0);
        store_s(g[(u + 2) % NSET], (u + 2) % NSET);
        mma(a[u], bf1, 1);
        read_b(bf0, (u + 1) % NSET, 0);
        __syncthreads();
      }
    }
    // tail (at most NSET + GD - 1 slabs): the same steps, guarded
    for (; base < nslab; base += NSET) {
#pragma unroll
      for (int u = 0; u < NSET; ++u) {
        const int sl = base + u;
        if (sl < nslab) {
          if (sl + GD < nslab) load_g(g[(u + GD) % NSET], sl + GD);
          if (sl + PD < nslab) load_a(a[(u + PD) % NSET], sl + PD);
          read_b(bf1, u, 1);
          mma(a[u], bf0, 0);
          if (sl + 2 < nslab) store_s(g[(u + 2) % NSET], (u + 2) % NSET);
          mma(a[u], bf1, 1);
          if (sl + 1 < nslab) read_b(bf0, (u + 1) % NSET, 0);
          __syncthreads();
        }
      }
    }

    // ---- the next tile's first slabs are requested before the epilogue runs
    const int cur_mat = mat;
    int cur_nt[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) cur_nt[ni] = nt[ni];
    if (t + 1 < t1) {
      set_tile(t + 1, wptr, nt, mat);
#pragma unroll
      for (int q = 0; q < GD; ++q)
        if (q < nslab) load_g(g[q], q);
#pragma unroll
      for (int q = 0; q < PD; ++q)
        if (q < nslab) load_a(a[q], q);
    }

    // ---- epilogue of tile t
    const int n_valid = p.n_valid[cur_mat];
    if (cur_mat == 1 || p.mode0 == 1) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        const int r = (mtile * MI + mi) * 16 + col;
        if (r >= p.R) continue;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
          const int v0 = cur_nt[ni] * 16 + grp * 4;
          float* o = p.out[cur_mat] + kpart * p.out_part_stride + (int64_t)r * p.ldo[cur_mat] + v0;
          if (v0 + 3 < n_valid && (p.ldo[cur_mat] & 3) == 0) {
            *reinterpret_cast<float4*>(o) = make_float4(acc[mi][ni][0], acc[mi][ni][1], acc[mi][ni][2], acc[mi][ni][3]);
          } else {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (v0 + i < n_valid) o[i] = acc[mi][ni][i];
          }
        }
      }
    } else {
      any_head = true;
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        // this lane's 4*NI logits of state row (mi, col), in increasing vocabulary order
        float x[NI * 4];
        float tmax = SPEC_NEG_INF;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int v = cur_nt[ni] * 16 + grp * 4 + i;
            const float xv = v < n_valid ? acc[mi][ni][i] : SPEC_NEG_INF;
            x[ni * 4 + i] = xv;
            tmax = fmaxf(tmax, xv);
          }
        const float new_m = fmaxf(run_m[mi], tmax);
        if (new_m > SPEC_NEG_INF) {
          float s = run_s[mi] * __expf(run_m[mi] - new_m);
#pragma unroll
          for (int e = 0; e < NI * 4; ++e) s += __expf(x[e] - new_m);
          run_s[mi] = s;
          run_m[mi] = new_m;
        }
        if (tmax > lv[mi][KT - 1]) {   // rare once the list has warmed up
#pragma unroll
          for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float xv = x[ni * 4 + i];
              if (xv > lv[mi][KT - 1]) {
                // a later vocabulary entry of equal value loses the tie: strict compares
                float cv = xv;
                int32_t ci = cur_nt[ni] * 16 + grp * 4 + i;
#pragma unroll
                for (int q = 0; q < KT; ++q) {
                  const bool gt = cv > lv[mi][q];
                  const float ov = lv[mi][q];
                  const int32_t oi = li[mi][q];
                  lv[mi][q] = gt ? cv : ov;
                  li[mi][q] = gt ? ci : oi;
                  cv = gt ? ov : cv;
                  ci = gt ? oi : ci;
                }
              }
            }
        }
      }
    }
  }

  if (!any_head) return;

  // ---- merge the 16 lane lists of every row (4 column groups x 4 waves) into the
  // workgroup's partial.  LDS aliases the slabs: the K loop ended on a barrier.
  constexpr int ROWS = 16 * MI;
  float* sv = reinterpret_cast<float*>(smem);                  // [256][MI][KT]
  int32_t* si = reinterpret_cast<int32_t*>(sv + 256 * MI * KT);
  float* sm = reinterpret_cast<float*>(si + 256 * MI * KT);    // [256][MI]
  float* ss = sm + 256 * MI;
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
    for (int q = 0; q < KT; ++q) {
      sv[(tid * MI + mi) * KT + q] = lv[mi][q];
      si[(tid * MI + mi) * KT + q] = li[mi][q];
    }
    sm[tid * MI + mi] = run_m[mi];
    ss[tid * MI + mi] = run_s[mi];
  }
  __syncthreads();
  for (int rl = tid; rl < ROWS; rl += 256) {
    const int r = mtile * ROWS + rl;
    if (r >= p.R) continue;
    const int mi = rl >> 4, c = rl & 15;
    float mx = SPEC_NEG_INF;
    for (int src = 0; src < 16; ++src) mx = fmaxf(mx, sm[((src >> 2) * 64 + (src & 3) * 16 + c) * MI + mi]);
    float s = 0.f;
    for (int src = 0; src < 16; ++src) {
      const int th = (src >> 2) * 64 + (src & 3) * 16 + c;
      const float m = sm[th * MI + mi];
      if (m > SPEC_NEG_INF) s += ss[th * MI + mi] * __expf(m - mx);
    }
    const int64_t slot = (int64_t)r * p.nparts + range;
    p.part.m[slot] = mx;
    p.part.s[slot] = s;
    // 16-way merge of sorted lists: only the heads compete; 4-bit read positions packed in one word
    uint64_t pos = 0;
    for (int j = 0; j < p.k_top; ++j) {
      float bv = SPEC_NEG_INF;
      int32_t bi = kIdxNone;
      int bsrc = 0;
      for (int src = 0; src < 16; ++src) {
        const int q = (int)((pos >> (4 * src)) & 15);
        if (q < KT) {
          const int th = (src >> 2) * 64 + (src & 3) * 16 + c;
          const float v = sv[(th * MI + mi) * KT + q];
          const int32_t i = si[(th * MI + mi) * KT + q];
          if (before(v, i, bv, bi)) { bv = v; bi = i; bsrc = src; }
        }
      }
      pos += (uint64_t)1 << (4 * bsrc);
      p.part.val[slot * p.k_top + j] = bv;
      p.part.idx[slot * p.k_top + j] = bi;
    }
  }
}

// Instruction pattern of one half of a slab in the wide kernel: N_MFMA matrix
// instructions with the half's memory instructions (LDS reads first, then global loads,
// then LDS writes) spread evenly behind them.  A wave issues in order, and a memory
// instruction takes several issue cycles: grouped in front of the matrix instructions
// they leave the matrix core idle (measured: 1320 cycles per slab against 980 when
// interleaved, 740 being the matrix work alone).
template <int N_MFMA, int N_DSR, int N_VMEM, int N_DSW>
__device__ __forceinline__ void interleave_half() {
  constexpr int TOTAL = N_DSR + N_VMEM + N_DSW;
#pragma unroll
  for (int i = 0; i < N_MFMA; ++i) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
#pragma unroll
    for (int j = i * TOTAL / N_MFMA; j < (i + 1) * TOTAL / N_MFMA; ++j) {
      if (j < N_DSR) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                // one LDS read
      else if (j < N_DSR + N_VMEM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);  // one global load
      else __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);                          // one LDS write
    }
  }
}

// Wide blocks: the same kernel built on v_mfma_f32_32x32x16_bf16.  One wave per SIMD can
// keep the matrix cores busy with the 32x32 instruction (measured: 2.1 PFLOP/s in a bare
// loop) but not with the 16x16 one (1.46 PFLOP/s: it needs a second wave per SIMD, and
// the wide tile leaves no registers for one).  The operands are gathered from the SAME
// tiled layout: a 32-row operand for K sub-step s of a 32-wide K step takes, for lane
// (row c = lane % 32, K half h = lane / 32), the 16-byte slot (2 s + h) * 16 + c % 16 of
// the 16-row tile pair member c / 16: four contiguous 256-byte pieces per wave load.
// Weights and states use the same assignment of K to lanes, which is all the contraction
// needs.  A lane then holds, for state row c of block mb, the logits of weight rows
// 32 nb + 4 h + 8 q + r (accumulator entry 4 q + r), in increasing vocabulary order.
// MB / NB = 32-row blocks of states per workgroup / of weight rows per wave.
template <int MB, int NB, int KT, bool VT>
__global__ __launch_bounds__(256, 1) void head_gemm32_kernel(GemmArgs p) {
  constexpr int MI = 2 * MB, NI = 2 * NB;  // in 16-row tiles of the layout
  // the tall block has 1.7x the matrix work per slab: two slabs ahead cover the same latency,
  // and the registers of the third go to the accumulators
  constexpr int PD = MB >= 5 ? 2 : ::specdraft::PD;
  constexpr int NSET = PD + 1;
  constexpr int GD = MB >= 5 ? 3 : ::specdraft::GD;
  static_assert(GD <= NSET && NSET >= 3, "register sets / LDS buffers are reused NSET slabs later");
  extern __shared__ __align__(16) unsigned char smem[];
  u32x4* ldsB = reinterpret_cast<u32x4*>(smem);  // [NSET][MI*KS*64]
  constexpr int SLAB = MI * KS * 64;             // slots per slab
  constexpr int SPT = SLAB / 256;                // staging slots per thread
  static_assert(SLAB % 256 == 0, "a slab is staged by whole passes of the workgroup");
  static_assert(KS == 2, "the K loop below is written for two K-steps per slab");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c32 = lane & 31, half = lane >> 5;

  // XCD-aware workgroup id: hardware places workgroup ids round-robin over 8 XCDs
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  if (seq >= p.chunk) return;
  const int wg = xcd * p.chunk + seq;
  if (wg >= p.m_tiles * p.n_ranges * p.ksplit) return;
  // K split (a projection alone, store epilogue): part kpart of a tile covers slabs [slab0, slab0 + nslab)
  const int kpart = wg % p.ksplit, wg2 = wg / p.ksplit;
  const int range = wg2 / p.m_tiles, mtile = wg2 - range * p.m_tiles;
  const int total_tiles = p.n_tiles[0] + p.n_tiles[1];
  const int t0 = (int)((int64_t)range * total_tiles / p.n_ranges);
  const int t1 = (int)((int64_t)(range + 1) * total_tiles / p.n_ranges);

  const int kt = p.kt;
  const int slab0 = (int)((int64_t)kpart * (kt / KS) / p.ksplit);
  const int nslab = (int)((int64_t)(kpart + 1) * (kt / KS) / p.ksplit) - slab0;
  // staging sources of this thread (the same for every tile of the range)
  const u32x4* sptr[SPT];
#pragma unroll
  for (int s = 0; s < SPT; ++s) {
    const int i = s * 256 + tid;
    const int mtl = i / (KS * 64), rem = i % (KS * 64);
    const int mt = min(mtile * MI + mtl, p.mt_total - 1);
    sptr[s] = p.b + (int64_t)mt * kt * 64 + (int64_t)slab0 * KS * 64 + rem;
  }

  // weight fragment pointers of this wave for a given tile of the list
  // VT (variable tile): a tile holds p.ts <= 4 * NI 16-row weight tiles instead of 4 * NI; wave w
  // owns tiles [w * NI, (w + 1) * NI) of it.  A 32-row block past the tile's end is masked in the
  // epilogue; its loads repeat the
  // tile's last 16 rows (lines another wave of the workgroup requests at the same time: no
  // extra HBM traffic, and short tiles are only planned where HBM is the bound).
  const u32x4* wptr[NB];
  auto set_tile = [&](int t, const u32x4* (&wp)[NB], int (&ntv)[NB], int& mat, int& tend) {
    mat = t >= p.n_tiles[0] ? 1 : 0;
    const int ntile = t - (mat ? p.n_tiles[0] : 0);
    const int ts = VT ? p.ts : 4 * NI;
    tend = VT ? min((ntile + 1) * ts, p.nt_total[mat]) : p.nt_total[mat];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
      ntv[nb] = ntile * ts + wave * NI + 2 * nb;  // first 16-row tile of the block
      const int ntc = min(ntv[nb] + (c32 >> 4), tend - 1);
      wp[nb] = p.w[mat] + (int64_t)ntc * kt * 64 + (int64_t)slab0 * KS * 64 + half * 16 + (c32 & 15);
    }
  };

  // Rotating register sets: weight fragments a[], state slots g[].
  u32x4 a[NSET][NB][2 * KS], g[NSET][SPT];
  auto load_g = [&](u32x4 (&gs)[SPT], int sl) {
    const int64_t off = (int64_t)sl * KS * 64;
#pragma unroll
    for (int s = 0; s < SPT; ++s) gs[s] = sptr[s][off];
  };
  auto load_a1 = [&](u32x4 (&aw)[NB][2 * KS], int sl, int nb) {
    const int64_t off = (int64_t)sl * KS * 64;
#pragma unroll
    for (int q = 0; q < 2 * KS; ++q) {  // q = 2 * K-step + sub-step
      // one block of state rows (MB == 2 serves <= 64 rows): nobody shares the weight stream, it need not stay cached
      if constexpr (MB == 2) aw[nb][q] = __builtin_nontemporal_load(wptr[nb] + off + q * 32);
      else aw[nb][q] = wptr[nb][off + q * 32];
    }
  };
  auto load_a = [&](u32x4 (&aw)[NB][2 * KS], int sl) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) load_a1(aw, sl, nb);
  };
  auto store_s = [&](const u32x4 (&gs)[SPT], int buf) {
#pragma unroll
    for (int s = 0; s < SPT; ++s) ldsB[buf * SLAB + s * 256 + tid] = gs[s];
  };

  // running softmax / top-k state of this lane, per state row (mi, col)
  float run_m[MB], run_s[MB], lv[MB][KT];
  int32_t li[MB][KT];
#pragma unroll
  for (int mi = 0; mi < MB; ++mi) {
    run_m[mi] = SPEC_NEG_INF;
    run_s[mi] = 0.f;
#pragma unroll
    for (int q = 0; q < KT; ++q) { lv[mi][q] = SPEC_NEG_INF; li[mi][q] = kIdxNone; }
  }
  bool any_head = false;

  int nt[NB], mat = 0, tend = 0;
  set_tile(t0, wptr, nt, mat, tend);
#pragma unroll
  for (int q = 0; q < GD; ++q)
    if (q < nslab) load_g(g[q], q);
#pragma unroll
  for (int q = 0; q < PD; ++q)
    if (q < nslab) load_a(a[q], q);

  for (int t = t0; t < t1; ++t) {
    f32x16 acc[MB][NB];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[mb][nb][e] = 0.f;
    // state operands of one 32-wide K step: [sub-step][block]
    auto read_b = [&](u32x4 (&bf)[2 * MB], int buf, int ts) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
          bf[s * MB + mb] =
              ldsB[buf * SLAB + ((2 * mb + (c32 >> 4)) * KS + ts) * 64 + (2 * s + half) * 16 + (c32 & 15)];
    };
    auto mma = [&](const u32x4 (&aw)[NB][2 * KS], const u32x4 (&bf)[2 * MB], int ts) {
#pragma unroll
      for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int mb = 0; mb < MB; ++mb)
            acc[mb][nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, aw[nb][2 * ts + s]),
                                                                  __builtin_bit_cast(bf16x8, bf[s * MB + mb]),
                                                                  acc[mb][nb], 0, 0, 0);
    };

    // ---- K loop (slab sl uses register set and LDS buffer sl % NSET; the loop is
    // unrolled NSET times so every index is a constant)
    store_s(g[0], 0);
    if (nslab > 1) store_s(g[1], 1);
    __syncthreads();
    u32x4 bf0[2 * MB], bf1[2 * MB];
    read_b(bf0, 0, 0);
    int base = 0;
    // steady state (whole groups of NSET slabs): no branches inside, so the compiler's
    // wait counters see straight-line code and let all the loads stay in flight.  Loads
    // that would run past the tile's last slab fetch that slab again (nobody uses them).
    for (; base + NSET <= nslab; base += NSET) {
#pragma unroll
      for (int u = 0; u < NSET; ++u) {
        const int sl_g = min(base + u + GD, nslab - 1), sl_a = min(base + u + PD, nslab - 1);
        // first half: K step 0 of the slab; behind its matrix instructions: the state
        // operands of K step 1, the state slots GD slabs ahead, the first weight block PD ahead
        read_b(bf1, u, 1);
        load_g(g[(u + GD) % NSET], sl_g);
        load_a1(a[(u + PD) % NSET], sl_a, 0);
        mma(a[u], bf0, 0);
        interleave_half<2 * NB * MB, 2 * MB, SPT + 2 * KS, 0>();
        __builtin_amdgcn_sched_barrier(0);
        // second half: K step 1; behind it: the next slab's first state operands, the
        // other weight blocks, the copy of the slab two ahead into LDS
        read_b(bf0, (u + 1) % NSET, 0);
#pragma unroll
        for (int nb = 1; nb < NB; ++nb) load_a1(a[(u + PD) % NSET], sl_a, nb);
        store_s(g[(u + 2) % NSET], (u + 2) % NSET);
        mma(a[u], bf1, 1);
        interleave_half<2 * NB * MB, 2 * MB, (NB - 1) * 2 * KS, SPT>();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
      }
    }
    // tail (fewer than NSET slabs): the same steps, guarded
    for (; base < nslab; base += NSET) {
#pragma unroll
      for (int u = 0; u < NSET; ++u) {
        const int sl = base + u;
        if (sl < nslab) {
          if (sl + GD < nslab) load_g(g[(u + GD) % NSET], sl + GD);
          if (sl + PD < nslab) load_a(a[(u + PD) % NSET], sl + PD);
          read_b(bf1, u, 1);
          __builtin_amdgcn_sched_barrier(0);
          mma(a[u], bf0, 0);
          __builtin_amdgcn_sched_barrier(0);
          if (sl + 2 < nslab) store_s(g[(u + 2) % NSET], (u + 2) % NSET);
          if (sl + 1 < nslab) read_b(bf0, (u + 1) % NSET, 0);
          __builtin_amdgcn_sched_barrier(0);
          mma(a[u], bf1, 1);
          __builtin_amdgcn_sched_barrier(0);
          __syncthreads();
        }
      }
    }

    // ---- the next tile's first slabs are requested before the epilogue runs
    const int cur_mat = mat, cur_end = tend;
    int cur_nt[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) cur_nt[nb] = nt[nb];
    if (t + 1 < t1) {
      set_tile(t + 1, wptr, nt, mat, tend);
#pragma unroll
      for (int q = 0; q < GD; ++q)
        if (q < nslab) load_g(g[q], q);
#pragma unroll
      for (int q = 0; q < PD; ++q)
        if (q < nslab) load_a(a[q], q);
    }

    // ---- epilogue of tile t
    // (variable tile: rows past the tile's end are another tile's)
    const int n_valid = VT ? min(p.n_valid[cur_mat], cur_end * 16) : p.n_valid[cur_mat];
    if (cur_mat == 1 || p.mode0 == 1) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        const int r = (mtile * MB + mb) * 32 + c32;
        if (r >= p.R) continue;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int v0 = cur_nt[nb] * 16 + half * 4 + 8 * q;
            float* o = p.out[cur_mat] + kpart * p.out_part_stride + (int64_t)r * p.ldo[cur_mat] + v0;
            if (v0 + 3 < n_valid && (p.ldo[cur_mat] & 3) == 0) {
              *reinterpret_cast<float4*>(o) = make_float4(acc[mb][nb][4 * q], acc[mb][nb][4 * q + 1],
                                                          acc[mb][nb][4 * q + 2], acc[mb][nb][4 * q + 3]);
            } else {
#pragma unroll
              for (int i = 0; i < 4; ++i)
                if (v0 + i < n_valid) o[i] = acc[mb][nb][4 * q + i];
            }
          }
      }
    } else {
      any_head = true;
    }
    // (a wave whose rows all lie past the tile's end has nothing to add)
    if (cur_mat == 0 && p.mode0 == 0 && (!VT || cur_nt[0] < cur_end)) {
      // only a block that reaches past the end of the tile or of the vocabulary needs the validity mask
      const bool edge = (cur_nt[NB - 1] + 2) * 16 > n_valid;
      constexpr float kLog2e = 1.4426950408889634f;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        // this lane's 16*NB logits of state row (mb, c32), in increasing vocabulary order
        float x[NB * 16];
        float tmax = SPEC_NEG_INF;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int v = cur_nt[nb] * 16 + half * 4 + 8 * (e >> 2) + (e & 3);
            const float xv = (!edge || v < n_valid) ? acc[mb][nb][e] : SPEC_NEG_INF;
            x[nb * 16 + e] = xv;
            tmax = fmaxf(tmax, xv);
          }
        const float new_m = fmaxf(run_m[mb], tmax);
        if (new_m > SPEC_NEG_INF) {
          // exp(x - m) as exp2(x * log2(e) - m * log2(e)): one fused multiply-add per logit
          const float ml = new_m * kLog2e;
          float s = run_s[mb] * __builtin_amdgcn_exp2f((run_m[mb] - new_m) * kLog2e);
#pragma unroll
          for (int e = 0; e < NB * 16; ++e) s += __builtin_amdgcn_exp2f(__builtin_fmaf(x[e], kLog2e, -ml));
          run_s[mb] = s;
          run_m[mb] = new_m;
        }
        if (tmax > lv[mb][KT - 1]) {
          // Branch-free insertion of every logit.  A range is only a few tiles long, so
          // the lists never warm up: some lane of the wave takes a new entry for almost every
          // element, and an insertion guarded by a per-element branch makes the whole wave
          // walk it anyway (measured: 9k-21k cycles per tile against 3k-7k this way).
          // Strict compares: a later vocabulary entry of equal value loses the tie.
#pragma unroll
          for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
              const float xv = x[nb * 16 + e];
              const int32_t xi = cur_nt[nb] * 16 + half * 4 + 8 * (e >> 2) + (e & 3);
              bool c[KT];
#pragma unroll
              for (int q = 0; q < KT; ++q) c[q] = xv > lv[mb][q];
#pragma unroll
              for (int q = KT - 1; q >= 1; --q) {
                lv[mb][q] = c[q - 1] ? lv[mb][q - 1] : (c[q] ? xv : lv[mb][q]);
                li[mb][q] = c[q - 1] ? li[mb][q - 1] : (c[q] ? xi : li[mb][q]);
              }
              lv[mb][0] = c[0] ? xv : lv[mb][0];
              li[mb][0] = c[0] ? xi : li[mb][0];
            }
        }
      }
    }
  }

  if (!any_head) return;

  // ---- merge the 8 lane lists of every row (2 K halves x 4 waves) into the workgroup's
  // partial.  LDS aliases the slabs: the K loop ended on a barrier.  The lists go to LDS as
  // 64-bit keys, a row's 8 lists side by side (rows one key apart from a power of two: the
  // writers of a wave hit distinct banks); then 8 adjacent lanes take one row, each its own
  // list in registers, and softmax pieces and the k best are reduced over the 8 lanes on
  // DPP - 32 rows per pass of the workgroup.  (One thread per row walking the 8 lists in
  // LDS took 6-12k cycles at the end of a launch, 10 % of a single-tile launch.)
  constexpr int ROWS = 32 * MB;
  constexpr int RS = 8 * KT + 1;
  uint64_t* sk = reinterpret_cast<uint64_t*>(smem);            // [ROWS][RS]
  float* sm = reinterpret_cast<float*>(sk + ROWS * RS);        // [ROWS][8]
  float* ss = sm + ROWS * 8;
  {
    const int src = tid >> 5;   // this thread's place among the 8 that hold a row
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      const int rl = mb * 32 + c32;
#pragma unroll
      for (int q = 0; q < KT; ++q) sk[rl * RS + src * KT + q] = best_key(lv[mb][q], li[mb][q]);
      sm[rl * 8 + src] = run_m[mb];
      ss[rl * 8 + src] = run_s[mb];
    }
  }
  __syncthreads();
  const uint64_t kEmpty = best_key(SPEC_NEG_INF, kIdxNone);
#pragma unroll 1
  for (int pass = 0; pass < MB; ++pass) {
    const int rl = pass * 32 + (tid >> 3), s8 = tid & 7;
    const int r = mtile * ROWS + rl;
    const bool live = r < p.R;
    uint64_t hk[KT];
#pragma unroll
    for (int q = 0; q < KT; ++q) hk[q] = sk[rl * RS + s8 * KT + q];
    const float m = sm[rl * 8 + s8], s = ss[rl * 8 + s8];
    float mx = fmaxf(m, dpp_f<kDppXor1>(m));
    mx = fmaxf(mx, dpp_f<kDppXor2>(mx));
    mx = fmaxf(mx, dpp_f<kDppHalfMirror>(mx));
    float sum = m > SPEC_NEG_INF ? s * __expf(m - mx) : 0.f;
    sum += dpp_f<kDppXor1>(sum);
    sum += dpp_f<kDppXor2>(sum);
    sum += dpp_f<kDppHalfMirror>(sum);
    const int64_t slot = (int64_t)r * p.nparts + range;
    if (live && s8 == 0) {
      p.part.m[slot] = mx;
      p.part.s[slot] = sum;
    }
#pragma unroll
    for (int j = 0; j < KT; ++j) {
      if (j < p.k_top) {
        uint64_t best = key_step<kDppXor1>(hk[0]);
        best = key_step<kDppXor2>(best);
        best = key_step<kDppHalfMirror>(best);
        const bool won = hk[0] == best;   // the owner of the winner pops it
#pragma unroll
        for (int q = 0; q + 1 < KT; ++q) {
          const uint64_t up = opaque_key(hk[q + 1]);
          hk[q] = won ? up : hk[q];
        }
        hk[KT - 1] = won ? kEmpty : hk[KT - 1];
        if (live && s8 == j) {
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

static size_t gemm_smem(int mi, int kcap) {
  const size_t slabs = (size_t)NSET * mi * KS * 64 * 16;
  const size_t merge = (size_t)256 * mi * (kcap * 8 + 8);
  return slabs > merge ? slabs : merge;
}

// dry: only answer whether this instance exists and how much LDS it takes (no HIP call)
template <int MI, int NI, int KT>
static hipError_t launch_gemm_t(const GemmArgs& a, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop,
                                size_t* dry) {
  const size_t smem = gemm_smem(MI, KT);
  if (dry) { *dry = smem; return hipSuccess; }
  static bool attr_set = false;  // per instantiation
  if (!attr_set && smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(head_gemm_kernel<MI, NI, KT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipExtLaunchKernelGGL((head_gemm_kernel<MI, NI, KT>), dim3(a.chunk * 8), dim3(256), smem, st, ev_start, ev_stop, 0, a);
  return hipGetLastError();
}

template <int MB, int NB, int KT, bool VT>
static hipError_t launch_gemm32_t(const GemmArgs& a, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop,
                                  size_t* dry) {
  const size_t smem = gemm_smem(2 * MB, KT);
  if (dry) { *dry = smem; return hipSuccess; }
  static bool attr_set = false;  // per instantiation
  if (!attr_set && smem > 64 * 1024) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(head_gemm32_kernel<MB, NB, KT, VT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipExtLaunchKernelGGL((head_gemm32_kernel<MB, NB, KT, VT>), dim3(a.chunk * 8), dim3(256), smem, st, ev_start, ev_stop, 0,
                        a);
  return hipGetLastError();
}

hipError_t launch_head_gemm(const HeadJob& job, const GemmPlan& pl, hipStream_t st, hipEvent_t ev_start,
                            hipEvent_t ev_stop, size_t* dry) {
  GemmArgs a;
  memset(&a, 0, sizeof(a));
  int nm = 0;
  if (job.vt_head > 0) {
    a.w[nm] = static_cast<const u32x4*>(job.w_head);
    a.nt_total[nm] = job.vt_head;
    a.n_valid[nm] = job.n_head;
    a.n_tiles[nm] = plan_tiles(job.n_head, pl.ts);
    a.out[nm] = job.out_head;
    a.ldo[nm] = job.ld_head;
    a.mode0 = job.out_head ? 1 : 0;
    ++nm;
  }
  if (job.vt_proj > 0) {
    if (nm == 0) a.mode0 = 1;  // projection alone: it is matrix 0 with the store epilogue
    a.w[nm] = static_cast<const u32x4*>(job.w_proj);
    a.nt_total[nm] = job.vt_proj;
    a.n_valid[nm] = job.n_proj;
    a.n_tiles[nm] = plan_tiles(job.n_proj, pl.ts);
    a.out[nm] = job.out_proj;
    a.ldo[nm] = job.ld_proj;
    ++nm;
  }
  if (nm == 0) return hipErrorInvalidValue;
  a.kt = job.kt;
  a.b = static_cast<const u32x4*>(job.b_src);
  a.b_rowmajor = job.b_rowmajor;
  a.b_ld = job.b_ld;
  if (job.b_rowmajor && (pl.ni != 1 || (job.b_ld & 7))) return hipErrorInvalidValue;  // narrow kernel only
  a.R = job.R;
  a.mt_total = (job.R + 15) / 16;
  a.m_tiles = pl.m_tiles;
  a.n_ranges = pl.n_ranges;
  a.ts = pl.ts;
  a.ksplit = 1;
  if (pl.ksplit > 1) {
    // only a projection alone, with room for the parts
    if (job.vt_head > 0 || job.proj_part_stride <= 0 || (job.proj_part_stride & 3)) return hipErrorInvalidValue;
    a.ksplit = pl.ksplit;
    a.out_part_stride = job.proj_part_stride;
  }
  a.chunk = (pl.m_tiles * pl.n_ranges * pl.ksplit + 7) / 8;
  a.k_top = job.k_top;
  a.part = job.part;
  a.nparts = job.nparts;
  if (a.mode0 == 0 && job.k_top > pl.kcap) return hipErrorInvalidValue;
  const int key = pl.mi * 100 + pl.ni * 10 + pl.kcap;
  const bool vt = pl.ni == 4 && pl.ts != 16;  // wide kernel with short tiles
  switch (key) {
    case 2 * 100 + 1 * 10 + 8: return launch_gemm_t<2, 1, 8>(a, st, ev_start, ev_stop, dry);
    case 4 * 100 + 1 * 10 + 8: return launch_gemm_t<4, 1, 8>(a, st, ev_start, ev_stop, dry);
#define WIDE_CASE(MB_, KT_)                                                             \
    case (2 * MB_) * 100 + 4 * 10 + KT_:                                                \
      return vt ? launch_gemm32_t<MB_, 2, KT_, true>(a, st, ev_start, ev_stop, dry)      \
                : launch_gemm32_t<MB_, 2, KT_, false>(a, st, ev_start, ev_stop, dry);
    // 33..64 rows (always short tiles)
    case 4 * 100 + 4 * 10 + 2: return launch_gemm32_t<2, 2, 2, true>(a, st, ev_start, ev_stop, dry);
    case 4 * 100 + 4 * 10 + 4: return launch_gemm32_t<2, 2, 4, true>(a, st, ev_start, ev_stop, dry);
    case 4 * 100 + 4 * 10 + 6: return launch_gemm32_t<2, 2, 6, true>(a, st, ev_start, ev_stop, dry);
    case 4 * 100 + 4 * 10 + 8: return launch_gemm32_t<2, 2, 8, true>(a, st, ev_start, ev_stop, dry);
    WIDE_CASE(3, 2) WIDE_CASE(3, 3) WIDE_CASE(3, 4) WIDE_CASE(3, 6) WIDE_CASE(3, 8)
    WIDE_CASE(4, 2) WIDE_CASE(4, 3) WIDE_CASE(4, 4)
    WIDE_CASE(5, 2) WIDE_CASE(5, 3) WIDE_CASE(5, 4)
#undef WIDE_CASE
    default: return hipErrorInvalidValue;
  }
}

}  // namespace specdraft
