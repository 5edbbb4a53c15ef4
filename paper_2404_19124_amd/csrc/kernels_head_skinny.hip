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

#include "head_skinny_body.h"

namespace specdraft {

bool skinny_fits(int R, int kt) {
  if (R < 1 || R > 16) return false;
  if ((kt + kSkinnyWaves - 1) / kSkinnyWaves > kSkinnySteps) return false;
  return (size_t)R * kt * 4 * 16 <= kSkinnyLdsB;
}
int skinny_grid(int n_cu) { return n_cu > 0 ? n_cu : 256; }

template <int NS, int DEPTH, bool EXACT>
__global__ __launch_bounds__(kSkinnyWaves * 64) void head_skinny_kernel(HeadJob p) {
  extern __shared__ __align__(16) unsigned char smem[];
  // the first tiles' weights are requested before anything else so that the stream is
  // already in flight while the states load
  u32x4 a[DEPTH][NS];
  skinny_prefetch<NS, DEPTH, EXACT>(p, blockIdx.x, gridDim.x, a);
  skinny_run<NS, DEPTH, EXACT>(p, blockIdx.x, gridDim.x, a, smem);
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

int skinny_fold_rows(int D) {
  constexpr int NT = kSkinnyWaves * 64;
  return (D > 0 && D % 512 == 0 && D / 8 <= NT) ? NT / (D / 8) : 0;
}

size_t skinny_lds_bytes(int R, int kt) { return skinny_state_bytes(R, kt) + kSkinnyLdsP; }

hipError_t launch_head_skinny(const HeadJob& job, int n_cu, hipStream_t st, hipEvent_t ev_start, hipEvent_t ev_stop) {
  const size_t smem = skinny_lds_bytes(job.R, job.kt);
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
