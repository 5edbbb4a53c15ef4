// Internal declarations shared by the HIP translation units of libspecdraft.
// Not part of the public boundary (that is include/spec.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace specdraft {

constexpr int kMaxTopK = 8;       // = SPEC_MAX_TOPK
constexpr int kMaxStages = 8;     // = SPEC_MAX_STAGES
constexpr int kMaxLeaves = 4096;  // = SPEC_MAX_LEAVES

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
// 16 raw bytes as a native vector (HIP's uint4 is a struct: copies of it can become
// memcpy calls that keep small arrays out of registers)
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// ---------------------------------------------------------------------------
// Tiled ("packed") bf16 layout.  A row-major matrix X[N][K] (K % 32 == 0) is
// stored as fragments of 16 rows x 32 columns, each fragment being exactly the
// per-lane operand order of v_mfma_f32_16x16x32_bf16:
//     slot(nt, t, lane) = 8 consecutive bf16 = X[nt*16 + lane%16][t*32 + (lane/16)*8 .. +8)
//     address (in 16-byte slots) = (nt * (K/32) + t) * 64 + lane
// so that a wave reads one fragment as one fully coalesced 1 KiB access.  Rows
// beyond N are zero (weights) or unspecified (states).
// ---------------------------------------------------------------------------

// Partial result of a head contraction for one (row, part): the running maximum
// and sum of exponentials of the logits seen by that part, and its k largest
// logits with their vocabulary indices (descending, ties by smaller index).
// Storage: m, s at [row * nparts + part]; val, idx at [(row * nparts + part) * k + j].
struct Partials {
  float* m;
  float* s;
  float* val;
  int32_t* idx;
};

// ---- packing --------------------------------------------------------------
// src row-major [n_rows][k] bf16 -> dst packed with ceil(n_rows/16) row tiles.
hipError_t launch_pack_bf16(const void* src, void* dst, int n_rows, int k, bool zero_pad, hipStream_t st);

// ---- contraction, bf16 on the matrix cores --------------------------------
// Optional prologue of the streaming kernel for the FIRST stage of a draft with one or two
// sequences: every workgroup computes the stage's state rows itself, straight into its LDS,
//   state_r = GELU(LayerNorm(w_s * pz[r] + w_e * Emb[tok_r]))  (Sec. 3.1),
// instead of reading them from a stage kernel's output, which removes a launch from the serial
// chain of a batch-1 step.  The few KB it reads arrive behind the weight tiles already
// requested (loads complete in order), i.e. when the weight ring has landed: one such round trip
// is free, because the stream is bound by HBM and the matrix cores catch up; a chain of them is
// not (measured: later stages, whose tokens first need a merge and whose rows take several
// rounds, lose 11-30 us this way and keep their stage kernel).
struct FoldJob {
  int enabled;
  int D, V;
  const float* pz;           // [R][D] projected states of the base model, as pz_parts partial sums
  int pz_parts;
  int64_t pz_part_stride;
  const int32_t* tok;        // [R] token of every row (the last sampled tokens)
  const void* emb;           // [V][D] bf16
  const float* gamma;
  const float* beta;
  float w_s, w_e, eps;
};

struct HeadJob {
  // weights (packed): `n_head` valid rows in `vt_head` tiles, then optionally a
  // second matrix (the next stage's projection) of `n_proj` rows in `vt_proj` tiles.
  const void* w_head;
  int vt_head, n_head;
  const void* w_proj;
  int vt_proj, n_proj;
  int kt;                 // K / 32
  // states: R rows; packed (one or more 16-row tiles) or row-major bf16 [R][ld]
  const void* b_src;
  int b_rowmajor, b_ld, R;
  // head epilogue: top-k partials (k_top entries) unless out_head != nullptr,
  // in which case raw logits are stored to out_head[r * ld_head + v]
  int k_top;
  Partials part;
  int nparts;
  float* out_head;
  int64_t ld_head;
  // projection epilogue: out_proj[r * ld_proj + d]
  float* out_proj;
  int64_t ld_proj;
  // a projection launched alone may be split along K (GemmPlan::ksplit): part q holds the sum over
  // its K range at out_proj + q * proj_part_stride, and the consumer adds the parts in order
  int64_t proj_part_stride;
  FoldJob fold;           // streaming kernel only
};

// Rows <= 16: one persistent workgroup per CU, K split over its 16 waves,
// weights streamed tile by tile straight into registers.  nparts = grid size.
bool skinny_fits(int R, int kt);
int skinny_grid(int n_cu);
size_t skinny_lds_bytes(int R, int kt);   // dynamic LDS of one workgroup
int skinny_fold_rows(int D);              // rows a FoldJob may have for inner width D (0: none)
// ev_start / ev_stop (may be null) receive the kernel's own begin / end timestamps.
hipError_t launch_head_skinny(const HeadJob& job, int n_cu, hipStream_t st, hipEvent_t ev_start = nullptr,
                              hipEvent_t ev_stop = nullptr);

// Any number of rows: workgroups of (16*mi state rows) x (64*ni weight rows) tiles, each
// persistent over one of n_ranges contiguous ranges of the weight-row tiles.  Head
// (top-k partials, one part per range that holds head tiles; or store) and, if present,
// the projection (store) in one launch.
struct GemmPlan {
  int mi, ni;        // fragments per wave in M (state rows) and N (weight rows)
  int ts;            // 16-row weight tiles per workgroup tile (<= 4 * ni; fewer = some waves' rows masked)
  int kcap;          // capacity of the per-lane top-k lists (>= k_top)
  int m_tiles;       // blocks of state rows
  int n_ranges;      // ranges of weight-row tiles
  int nparts;        // ranges that hold head tiles = parts per row
  int ksplit;        // parts of K (> 1 only for a projection alone)
};
constexpr int kMaxKSplit = 4;
GemmPlan plan_gemm(int R, int k_top, int n_head, int n_proj, int kt, int n_cu);
// true: the head and the next projection are cheaper as two launches than as one
bool plan_projection_apart(int R, int k_top, int n_head, int n_proj, int kt, int n_cu);
// dry != nullptr: nothing is launched (no HIP call at all); the result says whether a kernel
// instance exists for the plan, and *dry receives its LDS bytes.
hipError_t launch_head_gemm(const HeadJob& job, const GemmPlan& plan, hipStream_t st, hipEvent_t ev_start = nullptr,
                            hipEvent_t ev_stop = nullptr, size_t* dry = nullptr);

// ---- contraction, float32 (correctness configuration) ---------------------
// out[r * ldo + v] = sum_k a[r * lda + k] * w[v * ldw + k]
hipError_t launch_gemm_f32(const float* a, int64_t lda, const float* w, int64_t ldw, float* out, int64_t ldo,
                           int R, int N, int K, hipStream_t st);
// one partial per row from materialised logits [R][ld]
hipError_t launch_row_topk_f32(const float* logits, int64_t ld, int R, int V, int k_top, Partials part,
                               hipStream_t st);
// logp[r][v] = logits[r][v] - logsumexp(logits[r])   (in place allowed)
hipError_t launch_row_log_softmax(const float* logits, float* logp, int64_t ld, int R, int V, hipStream_t st);

// ---- measurement aid: plain copy of n16 16-byte words -----------------------
hipError_t launch_copy_probe(const void* src, void* dst, int64_t n16, hipStream_t st);

// ---- stage: merge of the previous head's partials + gather + mix + LN + GELU
struct StageJob {
  int stage;               // 0-based
  int R;                   // child rows of this stage
  int k_prev;              // top_k of the previous stage (1 for stage 0)
  int xcd_rows;            // 1: the 16 rows of a state tile run on one XCD (packed bf16 states, many rows)
  int D;
  int bf16;                // weight / state storage type
  // previous head (stage > 0)
  Partials part;
  int nparts, V;
  int32_t* prev_tok;       // [R/k_prev][k_prev] out
  float* prev_logp;        // same layout, out
  float* prev_lse;         // [R/k_prev] out
  const int32_t* last_tok; // stage 0: [R]
  const float* pz;         // [R/k_prev][D] projected parent state ...
  int pz_parts;            // ... as the sum of this many partial projections (0 or 1: a single one),
  int64_t pz_part_stride;  // pz_part_stride floats apart
  const void* emb;         // [V][D]
  const float* gamma;
  const float* beta;
  float w_s, w_e, eps;
  void* state_out;         // bf16: packed tiles; f32: row-major [R][D]
  void* state_dbg;         // optional row-major [R][D] copy in the storage type
  // Per-sequence trees (Sec. 4.2, 5: own branching per request): row r hangs under row row_parent[r] of
  // the previous stage (stage 0: under sequence row_parent[r]) as its row_rank[r]-th child; k_prev is then
  // the width of the previous stage's tables.  Null: the uniform tree, parent = r / k_prev, rank = r % k_prev.
  const int32_t* row_parent;
  const int32_t* row_rank;
};
hipError_t launch_stage(const StageJob& job, hipStream_t st);

// ---- tree: merge of the last head + leaf scores + top-B ----------------------
struct TreeJob {
  int batch, n, B, L;
  int B_pad;               // candidate slots per sequence in the outputs (>= B; slots past a sequence's B are padding)
  int kstride[kMaxStages]; // width of stage i's tables and of its head's partial lists (uniform tree: = top_k[i])
  // Per-sequence trees: seq_desc[q * (2 n + 1) + ..] = { k_0 .. k_{n-1}, first row of q at stage 0 .. n-1, B_q };
  // B_q = 0: the sequence has no rows and gets padding only.  Null: the uniform tree below.
  const int32_t* seq_desc;
  int top_k[kMaxStages];
  Partials part;           // last head
  int nparts;
  // per-stage tables [R_i][k_i], concatenated; offsets in elements
  int32_t* tok;
  float* logp;
  float* lse;              // [sum R_i]
  int64_t off[kMaxStages]; // element offset of stage i in tok / logp
  int64_t row_off[kMaxStages];
  int32_t* cand_tokens;
  float* cand_scores;
  int32_t* cand_leaf;
};
hipError_t launch_tree(const TreeJob& job, hipStream_t st);

// ---- verify ----------------------------------------------------------------
// n_cand (dev [batch], may be null = every sequence has B candidates): sequence q has n_cand[q] candidates;
// only rows (q, c < max(n_cand[q], 1), p) are scanned, and of a sequence without candidates only p = 0 (the
// base model's own next token); rows not scanned get greedy = -1.
hipError_t launch_argmax_rows(const void* logits, int bf16, int64_t rows, int V, int B, int n1, const int32_t* n_cand,
                              int32_t* greedy, hipStream_t st);
hipError_t launch_accept(const int32_t* greedy, const int32_t* cand, const int32_t* n_cand, int batch, int B, int n,
                         int32_t* accept_len, int32_t* best_cand, int32_t* out_tokens, int32_t* n_out,
                         int32_t* accept_all, hipStream_t st);

// ---- token tree of the candidates, hand-over to the next step ----------------
constexpr int kMaxTreeItems = 4096;  // B * n_predict per sequence (3 ints of LDS each)
hipError_t launch_tree_meta(const int32_t* cand, int batch, int B, int n, int32_t* node_tok, int32_t* node_parent,
                            int32_t* node_depth, int32_t* n_nodes, int32_t* cand_node, uint8_t* mask, hipStream_t st);
hipError_t launch_advance(const void* hidden, int64_t row_bytes, int batch, int B, int n, const int32_t* best,
                          const int32_t* accept, const int32_t* out_tokens, void* next_state, int32_t* next_tok,
                          hipStream_t st);

}  // namespace specdraft
