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
//    the CU.  At the end the workgroup writes one partial per row;
//  * at batch 1 the launch ends with a closing step (TailJob): the workgroup that finishes last merges
//    everybody's partials and computes the next stage's rows (or the tree step), so that no launch of
//    its own sits between two heads.
#include <hip/hip_ext.h>

#include <cstring>

#include "head_skinny_body.h"
#include "stage_body.h"

namespace specdraft {

bool skinny_fits(int R, int kt) {
  if (R < 1 || R > 16) return false;
  if ((kt + kSkinnyWaves - 1) / kSkinnyWaves > kSkinnySteps) return false;
  return (size_t)R * kt * 4 * 16 <= kSkinnyLdsB;
}
int skinny_grid(int n_cu) { return n_cu > 0 ? n_cu : 256; }
bool tail_fits(int rows, int D) { return rows >= 1 && rows <= 16 && D % 8 == 0 && D <= 4096; }

// Counts this workgroup in (thread 0 only; the workgroup's stores have been acknowledged) and tells
// whether it completed the count.  Two levels, every word on a cache line of its own: arrivals on one
// word would serialise in the memory system.  The workgroup that completes a counter sets it back to
// zero, so the words are zero again when the launch ends.
__device__ __forceinline__ bool tail_count_in(unsigned* ctr) {
  const unsigned G = gridDim.x, groups = G < 16u ? G : 16u, g = blockIdx.x % groups;
  const unsigned size_g = (G - g + groups - 1) / groups;
  unsigned* cg = ctr + (1 + g) * 32;
  if (__hip_atomic_fetch_add(cg, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u != size_g) return false;
  __hip_atomic_store(cg, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (__hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + 1u != groups) return false;
  __hip_atomic_store(ctr, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return true;
}

// TAIL: the launch has a closing step (TailJob): results are stored at agent scope, every workgroup counts
// itself in, and the one that completes the count computes the next stage's rows (or the tree step) from
// everybody's results.  What the closing workgroup reads was written through to memory by stores that were
// acknowledged before their workgroup counted itself in, into buffers nobody has read since the launch began
// (no cache can hold a stale line of them); what it writes is read by the NEXT launch only.
template <int NS, int DEPTH, bool EXACT, bool TAIL>
__global__ __launch_bounds__(kSkinnyWaves * 64) void head_skinny_kernel(HeadJob p, TailJob t) {
  extern __shared__ __align__(16) unsigned char smem[];
  // the first tiles' weights are requested before anything else so that the stream is
  // already in flight while the states load
  u32x4 a[DEPTH][NS];
  skinny_prefetch<NS, DEPTH, EXACT>(p, blockIdx.x, gridDim.x, a);
  skinny_run<NS, DEPTH, EXACT, TAIL>(p, blockIdx.x, gridDim.x, a, smem);
  if (!TAIL) return;

  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  int* s_last = reinterpret_cast<int*>(smem);
  if (threadIdx.x == 0) *s_last = tail_count_in(t.counters) ? 1 : 0;
  __syncthreads();
  const bool last = *s_last != 0;
  __syncthreads();
  if (!last) return;

  constexpr int NT = kSkinnyWaves * 64;
  if (t.kind == 1) {
    float* lds = reinterpret_cast<float*>(smem);
    if (t.stage.D > 2048) stage_all_rows<2>(t.stage, lds);
    else stage_all_rows<1>(t.stage, lds);
  } else if (t.kind == 2) {
    float* sc = reinterpret_cast<float*>(smem);
    int* s_k = reinterpret_cast<int*>(sc + kMaxLeaves);
    int* s_kw = s_k + kMaxStages;
    int64_t* s_off = reinterpret_cast<int64_t*>(s_kw + kMaxStages);
    int64_t* s_rbase = s_off + kMaxStages;
    float* merge_lds = reinterpret_cast<float*>(s_rbase + kMaxStages);
    for (int q = 0; q < t.tree.batch; ++q) {
      TreeArgs ta;
      __syncthreads();
      tree_args_for_sequence(t.tree, q, ta, s_k, s_off, s_rbase, s_kw);
      __syncthreads();
      tree_body<NT, 4>(ta, q, s_k, s_off, s_rbase, s_kw, sc, merge_lds);
    }
  }
}

template <int NS, int DEPTH, bool EXACT>
static hipError_t launch_skinny_t(const HeadJob& job, const TailJob* tail, int grid, size_t smem, hipStream_t st,
                                  hipEvent_t ev_start, hipEvent_t ev_stop) {
  static bool attr_set[2] = {false, false};  // per instantiation
  const bool with_tail = tail != nullptr && tail->kind != 0;
  const void* fn = with_tail ? reinterpret_cast<const void*>(head_skinny_kernel<NS, DEPTH, EXACT, true>)
                             : reinterpret_cast<const void*>(head_skinny_kernel<NS, DEPTH, EXACT, false>);
  if (!attr_set[with_tail]) {
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kSkinnyLdsB + kSkinnyLdsP));
    if (e != hipSuccess) return e;
    attr_set[with_tail] = true;
  }
  if (with_tail) {
    hipExtLaunchKernelGGL((head_skinny_kernel<NS, DEPTH, EXACT, true>), dim3(grid), dim3(kSkinnyWaves * 64), smem, st,
                          ev_start, ev_stop, 0, job, *tail);
  } else {
    TailJob none;
    memset(&none, 0, sizeof(none));
    hipExtLaunchKernelGGL((head_skinny_kernel<NS, DEPTH, EXACT, false>), dim3(grid), dim3(kSkinnyWaves * 64), smem, st,
                          ev_start, ev_stop, 0, job, none);
  }
  return hipGetLastError();
}

size_t skinny_lds_bytes(int R, int kt) { return skinny_state_bytes(R, kt) + kSkinnyLdsP; }

hipError_t launch_head_skinny(const HeadJob& job, const TailJob* tail, int n_cu, hipStream_t st, hipEvent_t ev_start,
                              hipEvent_t ev_stop) {
  const size_t smem = skinny_lds_bytes(job.R, job.kt);
  const int grid = skinny_grid(n_cu);
  if (tail && tail->kind != 0 && !tail->counters) return hipErrorInvalidValue;
  // K = 512 * NS gets an exact instantiation with as many tiles in flight as 16 fragments allow
  switch (job.kt % kSkinnyWaves == 0 ? job.kt / kSkinnyWaves : 0) {
    case 4: return launch_skinny_t<4, 4, true>(job, tail, grid, smem, st, ev_start, ev_stop);
    case 6: return launch_skinny_t<6, 2, true>(job, tail, grid, smem, st, ev_start, ev_stop);
    case 8: return launch_skinny_t<8, 2, true>(job, tail, grid, smem, st, ev_start, ev_stop);
    case 10: return launch_skinny_t<10, 1, true>(job, tail, grid, smem, st, ev_start, ev_stop);
    case 16: return launch_skinny_t<16, 1, true>(job, tail, grid, smem, st, ev_start, ev_stop);
    default: return launch_skinny_t<kSkinnySteps, 1, false>(job, tail, grid, smem, st, ev_start, ev_stop);
  }
}

}  // namespace specdraft
