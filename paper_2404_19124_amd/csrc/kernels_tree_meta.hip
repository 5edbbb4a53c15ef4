// Token tree of a sequence's candidates and the hand-over to the next step
// (Sec. 3.1 of the paper: multi-candidate decoding with tree attention; the base model
// is stage 0 of the next draft).
#include "device_utils.h"
#include "spec_internal.h"

namespace specdraft {

// One workgroup per sequence.  Item i = (c, p) stands for the prefix cand[c, :p+1].
//   first[i] = the smallest c' whose prefix of the same length is equal -> item (c', p)
//   a prefix is a node where first[i] == i; nodes are numbered in item order.
// M = B * n <= kMaxTreeItems.  Dynamic LDS: 3 * M ints.
__global__ __launch_bounds__(256) void tree_meta_kernel(const int32_t* __restrict__ cand, int B, int n,
                                                        int32_t* node_tok, int32_t* node_parent, int32_t* node_depth,
                                                        int32_t* n_nodes, int32_t* cand_node, uint8_t* mask) {
  extern __shared__ int32_t lds[];
  const int M = B * n;
  int32_t* tok = lds;          // [M]
  int32_t* first = lds + M;    // [M]
  int32_t* nid = lds + 2 * M;  // [M] node number of item i's prefix
  const int q = blockIdx.x, tid = threadIdx.x;
  const int32_t* cq = cand + (int64_t)q * M;
  for (int i = tid; i < M; i += 256) tok[i] = cq[i];
  if (mask) {
    uint8_t* mq = mask + (int64_t)q * M * M;
    for (int64_t i = tid; i < (int64_t)M * M; i += 256) mq[i] = 0;
  }
  __syncthreads();
  for (int i = tid; i < M; i += 256) {
    const int c = i / n, p = i - c * n;
    int f = i;
    for (int c2 = 0; c2 < c; ++c2) {
      bool same = true;
      for (int j = 0; j <= p; ++j) same = same && tok[c2 * n + j] == tok[c * n + j];
      if (same) { f = c2 * n + p; break; }
    }
    first[i] = f;
  }
  __syncthreads();
  for (int i = tid; i < M; i += 256) {
    int before = 0;
    for (int j = 0; j < i; ++j) before += first[j] == j ? 1 : 0;
    nid[i] = before;   // valid where first[i] == i
  }
  __syncthreads();
  int total = 0;
  if (tid == 0) {
    for (int j = 0; j < M; ++j) total += first[j] == j ? 1 : 0;
    n_nodes[q] = total;
  }
  for (int i = tid; i < M; i += 256) {
    const int c = i / n, p = i - c * n;
    const int me = nid[first[i]];
    cand_node[(int64_t)q * M + i] = me;
    if (first[i] == i) {
      node_tok[(int64_t)q * M + me] = tok[i];
      node_depth[(int64_t)q * M + me] = p + 1;
      node_parent[(int64_t)q * M + me] = p == 0 ? -1 : nid[first[i - 1]];
      if (mask) {
        uint8_t* row = mask + ((int64_t)q * M + me) * M;
        for (int j = 0; j <= p; ++j) row[nid[first[c * n + j]]] = 1;
      }
    }
  }
  // entries past the last node
  __syncthreads();
  if (tid == 0) lds[0] = total;   // tok[] is no longer needed
  __syncthreads();
  const int N = lds[0];
  for (int i = N + tid; i < M; i += 256) {
    node_tok[(int64_t)q * M + i] = -1;
    node_parent[(int64_t)q * M + i] = -1;
    node_depth[(int64_t)q * M + i] = 0;
  }
}

hipError_t launch_tree_meta(const int32_t* cand, int batch, int B, int n, int32_t* node_tok, int32_t* node_parent,
                            int32_t* node_depth, int32_t* n_nodes, int32_t* cand_node, uint8_t* mask,
                            hipStream_t st) {
  const size_t smem = (size_t)3 * B * n * sizeof(int32_t);
  hipLaunchKernelGGL(tree_meta_kernel, dim3(batch), dim3(256), smem, st, cand, B, n, node_tok, node_parent, node_depth,
                     n_nodes, cand_node, mask);
  return hipGetLastError();
}

// next_state[q] = hidden[q, best[q], accept[q], :], next_tok[q] = out_tokens[q, accept[q]].
// Indices are clamped to their ranges (a corrupted accept length must not leave the tensor).
__global__ __launch_bounds__(256) void advance_kernel(const uint8_t* __restrict__ hidden, int64_t row_bytes, int B, int n,
                                                      const int32_t* best, const int32_t* accept,
                                                      const int32_t* out_tokens, uint8_t* next_state,
                                                      int32_t* next_tok) {
  const int q = blockIdx.x;
  const int c = min(max(best[q], 0), B - 1), a = min(max(accept[q], 0), n);
  const uint8_t* src = hidden + (((int64_t)q * B + c) * (n + 1) + a) * row_bytes;
  uint8_t* dst = next_state + (int64_t)q * row_bytes;
  if ((row_bytes & 15) == 0 && ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) == 0) {
    for (int64_t i = threadIdx.x; i < row_bytes / 16; i += 256)
      reinterpret_cast<u32x4*>(dst)[i] = reinterpret_cast<const u32x4*>(src)[i];
  } else {
    for (int64_t i = threadIdx.x; i < row_bytes; i += 256) dst[i] = src[i];
  }
  if (threadIdx.x == 0) next_tok[q] = out_tokens[(int64_t)q * (n + 1) + a];
}

hipError_t launch_advance(const void* hidden, int64_t row_bytes, int batch, int B, int n, const int32_t* best,
                          const int32_t* accept, const int32_t* out_tokens, void* next_state, int32_t* next_tok,
                          hipStream_t st) {
  hipLaunchKernelGGL(advance_kernel, dim3(batch), dim3(256), 0, st, static_cast<const uint8_t*>(hidden), row_bytes, B, n,
                     best, accept, out_tokens, static_cast<uint8_t*>(next_state), next_tok);
  return hipGetLastError();
}

}  // namespace specdraft
