// Whole draft (Sec. 3.1, 4.1 of the paper) in ONE launch, for the batch-1 regime in
// which every stage has at most 16 rows:
//   proj_1 | barrier | for each stage: [stage rows | barrier | head_i (+ proj_{i+1}) | barrier] | tree
// The phases are the bodies of the stand-alone kernels (head_skinny_body.h,
// stage_body.h); what the fusion buys on the serial chain of a bandwidth-bound step:
//  * no kernel boundaries: a boundary costs a drain, a launch and a cold start of the
//    weight stream, about ten times per draft;
//  * the first tiles of head_i's weights are requested BEFORE the barrier in front of
//    the head (by all but the few workgroups that compute a stage row: before the stage
//    phase), so the HBM stream is already running when the states
//    arrive (weights do not depend on anything computed in the launch).
//
// One workgroup of 16 waves per CU; all of them are resident at once (the launch asks
// for exactly one per CU and a CU holds one), which the barrier needs.  The barrier is a
// monotone device-wide counter: arrive with an atomic add, wait until it reaches the
// phase's target.  The wait is bounded by a wall-clock limit: if it expires (workgroups
// not co-resident, e.g. CUs masked off), the workgroup raises a flag in host-visible
// memory and leaves; every wave reaches the end of the kernel either way.
#include <hip/hip_ext.h>

#include "head_skinny_body.h"
#include "stage_body.h"

namespace specdraft {

// Head of dynamic LDS: the barrier's flag (the rest of the block keeps the contraction's
// buffers aligned).
constexpr size_t kFusedDescBytes = 256;

bool fused_fits(int max_rows, int kt_in, int kt, int n_cu) {
  if (n_cu < 1 || max_rows < 1 || max_rows > 16) return false;
  if (kt_in != kt) return false;                       // one K split for every contraction
  if (kt % kSkinnyWaves) return false;
  const int ns = kt / kSkinnyWaves;
  if (ns != 1 && ns != 2 && ns != 4 && ns != 6 && ns != 8) return false;
  return kFusedDescBytes + skinny_state_bytes(max_rows, kt) + kSkinnyLdsP <= kSkinnyLdsB + kSkinnyLdsP;
}

// Device-wide barrier over the G resident workgroups.  Returns false when the wait
// ran into its time limit (the caller then leaves the kernel).
//
// No cache is written back or invalidated here (an L2-wide operation per workgroup and
// barrier costs more than a whole phase).  Instead:
//  * what a phase hands to other workgroups is stored with agent-scope stores
//    (store_agent: written through to memory), and every wave waits for its stores to
//    be acknowledged before the workgroup arrives;
//  * every buffer handed over is written ONCE per launch and not read before that (one
//    set per stage), and the caches are clean of it when the launch starts, so no L1 or
//    L2 can hold a stale line: the first read after the barrier comes from memory;
//  * the arrival counter itself is only touched with agent-scope atomics.
//
// Arrivals on ONE counter would serialise in the memory system (256 atomics and 256
// pollers on one address take 10-20 us), so the barrier is a two-level tree over
// kBarrierGroups groups of workgroups (group = id mod kBarrierGroups), every word on a
// cache line of its own:
//   group counter  <- every workgroup of the group adds 1
//   root counter   <- the last arrival of each group adds 1
//   group flag     <- the last arrival at the root stores the barrier's number into every
//                     group's flag; the workgroups of a group poll their own flag.
// All words are monotone over the life of the model: barrier number e (counted from 1
// over all launches, modulo 2^32) completes group g at e * size(g) arrivals, the root
// at e * groups, and the flags at e.
constexpr int kBarrierGroups = 16;
constexpr int kBarrierLine = 32;  // words per 128-byte line
// words of the barrier block: line 0 = root, lines 1.. = group counters, then group flags
constexpr size_t kBarrierWords = (size_t)(1 + 2 * kBarrierGroups) * kBarrierLine;
size_t fused_barrier_bytes() { return kBarrierWords * sizeof(unsigned); }

__device__ __forceinline__ bool grid_barrier(unsigned* bar, unsigned epoch, unsigned long long limit_ticks,
                                             int* lds_flag) {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) {
    const unsigned G = gridDim.x, wg = blockIdx.x;
    const unsigned groups = G < (unsigned)kBarrierGroups ? G : (unsigned)kBarrierGroups;
    const unsigned g = wg % groups;
    const unsigned size_g = (G - g + groups - 1) / groups;
    unsigned* root = bar;
    unsigned* grp = bar + (1 + g) * kBarrierLine;
    unsigned* flags = bar + (1 + kBarrierGroups) * kBarrierLine;
    const unsigned old = __hip_atomic_fetch_add(grp, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old + 1u == epoch * size_g) {
      const unsigned oldr = __hip_atomic_fetch_add(root, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (oldr + 1u == epoch * groups) {
        for (unsigned h = 0; h < groups; ++h)
          __hip_atomic_store(flags + h * kBarrierLine, epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
    int ok = 1;
    const unsigned long long t0 = wall_clock64();
    while ((int)(__hip_atomic_load(flags + g * kBarrierLine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - epoch) < 0) {
      __builtin_amdgcn_s_sleep(1);
      if (wall_clock64() - t0 > limit_ticks) {
        ok = 0;
        break;
      }
    }
    *lds_flag = ok;
  }
  __syncthreads();
  return *lds_flag != 0;
}

// The phases are separate (not inlined) functions: each gets a register allocation of its
// own.  Inlined into one body, the compiler kept values of one phase alive through the
// others and spilled the prefetched weights.  Arguments of a device function arrive in
// vector registers, so the phases take only a few integers, make them scalar again, and
// read everything else from the kernel-argument segment (constant address space, scalar
// loads on demand; indexing the by-value kernel argument itself with run-time stage
// numbers would make the compiler copy the whole block to scratch).
typedef const __attribute__((address_space(4))) FusedJob* fused_job_ptr;
typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;

typedef const __attribute__((address_space(4))) unsigned char* const_byte_ptr;

// Only a kernel can ask for its argument segment (in a device function the builtin
// yields a null pointer); what a device function does receive is the pointer to the
// implicit arguments, which follow the explicit ones in the same segment.  The kernel
// measures the distance between the two and hands it to the phases.
__device__ __forceinline__ unsigned fused_job_distance() {
  return (unsigned)((const_byte_ptr)__builtin_amdgcn_implicitarg_ptr() -
                    (const_byte_ptr)__builtin_amdgcn_kernarg_segment_ptr());
}
__device__ __forceinline__ const FusedJob* fused_job_in_kernel() {
  return (const FusedJob*)((fused_job_ptr)__builtin_amdgcn_kernarg_segment_ptr());
}
__device__ __forceinline__ const FusedJob* fused_job(unsigned distance_v) {
  const unsigned distance = __builtin_amdgcn_readfirstlane(distance_v);
  return (const FusedJob*)((fused_job_ptr)((const_byte_ptr)__builtin_amdgcn_implicitarg_ptr() - distance));
}
__device__ __forceinline__ unsigned char* lds_at(unsigned offset_v) {
  return (unsigned char*)((lds_byte_ptr)(uintptr_t)__builtin_amdgcn_readfirstlane(offset_v));
}

// head[idx]: request the first tiles, wait at the barrier in front of the phase (idx > 0),
// run the contraction.  Returns 0 when the barrier wait ran out of time.
template <int NS, int DEPTH>
__device__ __attribute__((noinline)) int fused_head_phase(int idx_v, unsigned target_v, unsigned lds_v, unsigned job_v) {
  const int idx = __builtin_amdgcn_readfirstlane(idx_v);
  const unsigned target = __builtin_amdgcn_readfirstlane(target_v);
  unsigned char* smem = lds_at(lds_v);
  const FusedJob* J = fused_job(job_v);
  const HeadJob& p = J->head[idx];
  const int wg = blockIdx.x, G = gridDim.x;
  u32x4 a[DEPTH][NS];
  skinny_prefetch<NS, DEPTH, true>(p, wg, G, a);
  if (idx > 0) {
    if (!grid_barrier(J->barrier, target, J->timeout_ticks, reinterpret_cast<int*>(smem))) return 0;
  }
  skinny_run<NS, DEPTH, true, true>(p, wg, G, a, smem + kFusedDescBytes);
  return 1;
}

// the rows of stage i this workgroup owns (none for most workgroups)
__device__ __attribute__((noinline)) void fused_stage_phase(int i_v, unsigned lds_v, unsigned job_v) {
  const int i = __builtin_amdgcn_readfirstlane(i_v);
  unsigned char* smem = lds_at(lds_v);
  const StageJob& sj = fused_job(job_v)->stage[i];
  const int G = gridDim.x;
  for (int r = blockIdx.x; r < sj.R; r += G)
    stage_row<true, 1, kSkinnyWaves * 64, true>(sj, r, reinterpret_cast<float*>(smem + kFusedDescBytes));
}

__device__ __attribute__((noinline)) void fused_tree_phase(unsigned lds_v, unsigned job_v) {
  constexpr int NT = kSkinnyWaves * 64;
  unsigned char* work = lds_at(lds_v) + kFusedDescBytes;
  const FusedJob* J = fused_job(job_v);
  const TreeJob* tj = &J->tree;
  const int tid = opaque_tid(), n = J->n, batch = J->batch, G = gridDim.x;
  float* sc = reinterpret_cast<float*>(work);
  int* s_k = reinterpret_cast<int*>(sc + kMaxLeaves);
  int* s_kw = s_k + kMaxStages;
  int64_t* s_off = reinterpret_cast<int64_t*>(s_kw + kMaxStages);
  int64_t* s_rbase = s_off + kMaxStages;
  float* merge_lds = reinterpret_cast<float*>(s_rbase + kMaxStages);
  (void)tid;
  (void)n;
  for (int q = blockIdx.x; q < batch; q += G) {
    TreeArgs t;
    __syncthreads();
    tree_args_for_sequence(*tj, q, t, s_k, s_off, s_rbase, s_kw);
    __syncthreads();
    tree_body<NT, 4>(t, q, s_k, s_off, s_rbase, s_kw, sc, merge_lds);
  }
}

template <int NS, int DEPTH>
__global__ __launch_bounds__(kSkinnyWaves * 64) void draft_fused_kernel(FusedJob jarg) {
  extern __shared__ __align__(16) unsigned char smem[];
  (void)jarg;
  const FusedJob* J = fused_job_in_kernel();
  const unsigned job_at = fused_job_distance();
  const unsigned lds_base = (unsigned)(uintptr_t)((lds_byte_ptr)smem);
  const int wg = blockIdx.x;
  const int n = J->n, batch = J->batch;
  unsigned target = J->barrier_base;  // number of the last barrier completed before this launch
  // time stamps of workgroup 0 (phase boundaries), if asked for
  unsigned long long* clocks = J->clocks;
  const bool stamp = clocks != nullptr && wg == 0;  // uniform
  int nclk = 0;
#define SPEC_STAMP()                                                  \
  do {                                                                \
    if (stamp) {                                                      \
      if (threadIdx.x == 0) clocks[nclk] = wall_clock64();            \
    }                                                                 \
    ++nclk;                                                           \
  } while (0)
#define SPEC_FAIL()                                                   \
  do {                                                                \
    if (threadIdx.x == 0) *J->fail_flag = 1;                          \
    return;                                                           \
  } while (0)

  SPEC_STAMP();
  fused_head_phase<NS, DEPTH>(0, 0u, lds_base, job_at);  // proj_1 of the base model's state
  SPEC_STAMP();
  for (int i = 0; i < n; ++i) {
    // barrier behind the previous contraction
    ++target;
    if (!grid_barrier(J->barrier, target, J->timeout_ticks, reinterpret_cast<int*>(smem))) SPEC_FAIL();
    SPEC_STAMP();
    fused_stage_phase(i, lds_base, job_at);
    // (the head phase waits at the barrier behind the stage rows itself, with its first
    // tiles already requested)
    ++target;
    if (!fused_head_phase<NS, DEPTH>(i + 1, target, lds_base, job_at)) SPEC_FAIL();
    SPEC_STAMP();
  }
  ++target;
  if (!grid_barrier(J->barrier, target, J->timeout_ticks, reinterpret_cast<int*>(smem))) SPEC_FAIL();
  SPEC_STAMP();
  if (wg < batch) fused_tree_phase(lds_base, job_at);
  SPEC_STAMP();
#undef SPEC_STAMP
#undef SPEC_FAIL
}

template <int NS, int DEPTH>
static hipError_t launch_fused_t(const FusedJob& job, size_t smem, hipStream_t st, hipEvent_t ev_start,
                                 hipEvent_t ev_stop) {
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(draft_fused_kernel<NS, DEPTH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kSkinnyLdsB + kSkinnyLdsP));
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipExtLaunchKernelGGL((draft_fused_kernel<NS, DEPTH>), dim3(job.n_wg), dim3(kSkinnyWaves * 64), smem, st, ev_start,
                        ev_stop, 0, job);
  return hipGetLastError();
}

hipError_t launch_draft_fused(const FusedJob& job, int max_rows, hipStream_t st, hipEvent_t ev_start,
                              hipEvent_t ev_stop) {
  const int kt = job.head[0].kt;
  if (!fused_fits(max_rows, kt, job.head[1].kt, job.n_wg)) return hipErrorInvalidValue;
  size_t smem = kFusedDescBytes + skinny_state_bytes(max_rows, kt) + kSkinnyLdsP;
  switch (kt / kSkinnyWaves) {
    case 1: return launch_fused_t<1, 8>(job, smem, st, ev_start, ev_stop);
    case 2: return launch_fused_t<2, 8>(job, smem, st, ev_start, ev_stop);
    case 4: return launch_fused_t<4, 4>(job, smem, st, ev_start, ev_stop);
    case 6: return launch_fused_t<6, 2>(job, smem, st, ev_start, ev_stop);
    case 8: return launch_fused_t<8, 2>(job, smem, st, ev_start, ev_stop);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace specdraft
