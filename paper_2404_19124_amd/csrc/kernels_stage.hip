// Stage kernel (Sec. 3.1 of the paper): for every node of the current depth,
//   state = GELU(LayerNorm(w_s * (W s_parent) + w_e * Emb[token]))
// The token a node carries is the j-th best of its parent's head row; that row's
// partial results are merged here (every sibling repeats the small merge, which
// saves a separate launch on the latency-critical batch-1 chain).
#include "stage_body.h"

namespace specdraft {

// NCH = 8-element chunks per thread held in registers (D <= NCH * NT * 8).
template <bool BF16, int NCH, int NT>
__global__ __launch_bounds__(NT) void stage_kernel(StageJob j) {
  __shared__ float lds[32 + (NT / 256) * kMergeLds];
  int r = blockIdx.x;
  if (j.xcd_rows) {
    // Workgroup ids go round-robin over the 8 XCDs, and a row's state is stored as one 16-byte slot in
    // each of D / 8 lines that it shares with the other rows of its 16-row tile.  Rows of one tile on
    // eight XCDs leave every L2 with an eighth of each line to write back; here the 16 rows of a tile
    // run on one XCD, whose L2 puts the lines together (7B shape, 64 sequences: -7 us per step).
    const int xcd = blockIdx.x & 7, s = blockIdx.x >> 3;
    r = (((s >> 4) << 3) + xcd) * 16 + (s & 15);
    if (r >= j.R) return;
  }
  stage_row<BF16, NCH, NT>(j, r, lds);
}

template <bool BF16>
static hipError_t launch_stage_t(const StageJob& job, hipStream_t st) {
  const int nchunk = job.D / 8;
  // tile-per-XCD order: whole groups of 8 tiles, the workgroups past the last row leave at once
  const dim3 grid(job.xcd_rows ? (job.R + 127) / 128 * 128 : job.R);
  // 512 threads per row from D = 4096 on: the row's LayerNorm / GELU arithmetic is what a workgroup spends its
  // time on once its loads are back, and eight waves halve it (7B batch 1: -1 us per step; 7-stage chain: -3.6 us)
  if (nchunk <= 256) hipLaunchKernelGGL((stage_kernel<BF16, 1, 256>), grid, dim3(256), 0, st, job);
  else if (nchunk <= 512) hipLaunchKernelGGL((stage_kernel<BF16, 1, 512>), grid, dim3(512), 0, st, job);
  else if (nchunk <= 1024) hipLaunchKernelGGL((stage_kernel<BF16, 2, 512>), grid, dim3(512), 0, st, job);
  else if (nchunk <= 2048) hipLaunchKernelGGL((stage_kernel<BF16, 4, 512>), grid, dim3(512), 0, st, job);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_stage(const StageJob& job, hipStream_t st) {
  return job.bf16 ? launch_stage_t<true>(job, st) : launch_stage_t<false>(job, st);
}

// ---------------------------------------------------------------------------
// Tree kernel (Sec. 3.1, 4.1): merge the last head's partial results, score
// every leaf by the sum of its tokens' log-probabilities (added in stage order),
// keep the B best.  One workgroup per sequence.
// ---------------------------------------------------------------------------
// NT = 512: eight waves merge eight rows at a time and each wave may use 256 registers (the
// widest merges need more than the 128 a 1024-thread workgroup would leave).  NT = 1024 for
// last-stage top-k <= 4 (KWAVE = 4): sixteen rows per pass, one pass for the paper's trees.
template <int NT, int KWAVE>
__global__ __launch_bounds__(NT) void tree_kernel(TreeJob j) {
  __shared__ __align__(16) uint64_t sk[kMaxLeaves];
  __shared__ int s_k[kMaxStages], s_kw[kMaxStages];
  __shared__ int64_t s_off[kMaxStages], s_rbase[kMaxStages];
  __shared__ float merge_lds[kMergeLds * (NT / 256)];
  __shared__ int32_t c_tok[kMaxLeaves];
  __shared__ float c_logp[kMaxLeaves];
  TreeArgs a;
  tree_args_for_sequence(j, blockIdx.x, a, s_k, s_off, s_rbase, s_kw);
  // (no barrier here: a wave reads back only what it wrote itself until the merge in tree_body ends in one,
  // so it starts its loads while the later waves of the workgroup are still being launched)
  tree_body<NT, KWAVE>(a, blockIdx.x, s_k, s_off, s_rbase, s_kw, sk, merge_lds, c_tok, c_logp);
}

hipError_t launch_tree(const TreeJob& job, hipStream_t st) {
  // (per-sequence trees: the widest table decides the merge variant, rows_last is then an upper bound)
  const int kw_last = job.kstride[job.n - 1];
  const int rows_last = job.seq_desc ? kMaxLeaves : job.L / job.top_k[job.n - 1];
  if (kw_last <= 4 && rows_last > 8)
    hipLaunchKernelGGL((tree_kernel<1024, 4>), dim3(job.batch), dim3(1024), 0, st, job);
  else
    hipLaunchKernelGGL((tree_kernel<512, kMaxTopK>), dim3(job.batch), dim3(512), 0, st, job);
  return hipGetLastError();
}

}  // namespace specdraft
