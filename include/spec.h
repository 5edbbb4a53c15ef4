/* spec.h -- C ABI of the MI355X draft + verify library (libspecdraft.so).
 *
 * One speculative-decoding step of the combined token/embedding speculator of
 * arXiv 2404.19124:  spec_draft runs the n-stage MLP speculator and emits the
 * pruned candidate tree (Sec. 3.1, 4.1 of the paper); spec_verify compares the
 * base model's logits over the flattened candidates with the speculated tokens
 * and emits the accepted tokens plus one bonus token (Sec. 1, 3.1, 5).
 *
 * Conventions
 *  - Plain C.  No exception crosses the boundary.  Every entry point checks its
 *    arguments on the host and returns a negative status BEFORE any HIP call;
 *    the message is available from spec_last_error() (thread-local).
 *  - Pointers marked "dev" are device pointers on the current HIP device, owned
 *    by the caller.  Pointers marked "host" are ordinary host pointers.
 *  - spec_draft and spec_verify only enqueue work on `hip_stream` (a
 *    hipStream_t passed as void*; NULL is the default stream).  They never
 *    synchronise and never allocate.  Outputs are valid once the stream has
 *    reached the end of the enqueued work.
 *  - A HIP runtime failure is reported as SPEC_EHIP with the HIP error string.
 *  - All matrices are row-major with the last index contiguous.
 */
#ifndef SPEC_DRAFT_H_
#define SPEC_DRAFT_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPEC_MAX_STAGES 8      /* n_predict <= 8 (the paper uses 3, 5 and 7) */
#define SPEC_MAX_TOPK 8        /* branches per head <= 8 (the paper uses up to 6) */
#define SPEC_MAX_LEAVES 4096   /* prod(top_k) <= 4096 per sequence */
#define SPEC_STATIC_SCRATCH_BYTES (8 * 1024 * 1024) /* workspace of spec_draft_static, per GPU */

typedef struct spec_model spec_model_t; /* opaque: packed weights, descriptors, workspace */

typedef enum { SPEC_F32 = 0, SPEC_BF16 = 1 } spec_dtype_t;

typedef enum {
  SPEC_OK = 0,
  SPEC_EINVAL = -1, /* null pointer, value out of range */
  SPEC_ESHAPE = -2, /* sizes inconsistent with the model or with each other */
  SPEC_EDTYPE = -3, /* unknown or unsupported element type */
  SPEC_ENOMEM = -4, /* device allocation failed (spec_create only) */
  SPEC_EHIP = -5    /* HIP runtime error */
} spec_status_t;

/* Shape of the speculator (Sec. 3.1: n stages; Sec. 4: latent width; Sec. 4.2:
 * only the first stage's input width follows the base model). */
typedef struct {
  int32_t n_predict;    /* n: stages = speculated tokens per candidate, 1..SPEC_MAX_STAGES */
  int32_t emb_dim;      /* E: width of the base model's hidden vector (input of stage 1) */
  int32_t inner_dim;    /* D: latent width of the speculator */
  int32_t vocab;        /* V */
  int32_t weight_dtype; /* spec_dtype_t: storage type of projection / head / embedding
                           weights, of the input state and of the stage states.
                           SPEC_BF16 needs E and D to be multiples of 64,
                           SPEC_F32 needs D to be a multiple of 8. */
  float state_weight;   /* w_s: weight of the projected state in the pair (Sec. 4).  If
                           state_weight < 0 or emb_weight < 0 both take the closed form of the
                           50%-variance rule:  w_s = 0.5^(1/2n), w_e = sqrt(1 - 0.5^(1/n)). */
  float emb_weight;     /* w_e: weight of the token embedding in the pair */
  float ln_eps;         /* LayerNorm epsilon (inside the root); <= 0 selects 1e-5 */
  int32_t max_batch;    /* largest batch spec_draft will be called with (sizes the workspace) */
  int32_t max_top_k[SPEC_MAX_STAGES]; /* per stage, largest top_k[i] spec_draft will be called
                           with; entries 0..n_predict-1 in 1..SPEC_MAX_TOPK */
} spec_config_t;

/* Per-stage weights: host arrays of length n_predict holding dev pointers.
 *   proj[i]     [D, in_i]  (in_0 = E, else D)   weight_dtype   state projection W_i
 *   emb[i]      [V, D]                          weight_dtype   token embedding table
 *   head[i]     [V, D]                          weight_dtype   vocabulary head
 *   ln_gamma[i] [D], ln_beta[i] [D]             float32        LayerNorm affine
 * The paper ties nothing across stages (Sec. 3.1); passing the same pointer for
 * several stages gives its weight-tied (RNN) variant (stages given the same proj / head
 * pointer, with the same shape, share one library copy).
 * Ownership: proj and head are COPIED by spec_create into library-owned buffers
 * (for SPEC_BF16 in a tiled layout that matches the matrix-core operand order),
 * the caller may release them once spec_create has returned.  emb, ln_gamma and
 * ln_beta are BORROWED and must stay valid and unchanged until spec_destroy. */
typedef struct {
  const void* const* proj;
  const void* const* emb;
  const void* const* head;
  const float* const* ln_gamma;
  const float* const* ln_beta;
} spec_weights_t;

/* Optional per-stage intermediates for parity checks (all dev, caller-allocated,
 * each pointer may be NULL).  Stage i occupies rows [sum_{j<i} R_j, +R_i) with
 * R_i = batch * prod_{j<i} top_k[j]; rows are sequence-major, then by the ranks
 * chosen at the earlier stages (node r has children r*k_i + j). */
typedef struct {
  void* stage_state;  /* [sum R_i, D] weight_dtype: state of every node */
  int32_t* topk_tok;  /* concatenated per stage [R_i, k_i]: tokens, most likely first */
  float* topk_logp;   /* same layout: their log-probabilities */
  float* row_lse;     /* [sum R_i]: log-sum-exp of every row's logits */
} spec_debug_t;

/* Builds a model: validates, copies / tiles proj and head, allocates the
 * workspace for (max_batch, max_top_k).  Uses `hip_stream` for the copies and
 * synchronises it before returning.  *out is set only on SPEC_OK. */
spec_status_t spec_create(const spec_config_t* cfg /* host */, const spec_weights_t* w /* host */,
                          void* hip_stream, spec_model_t** out /* host */);

/* Releases everything spec_create allocated.  NULL is allowed.  The caller must
 * make sure no enqueued work still uses the model. */
void spec_destroy(spec_model_t* m);

/* DRAFT (Sec. 3.1, 4.1).  For each of `batch` sequences: starting from the base
 * model's last hidden vector and the token it just sampled, stage i computes
 *     state_i = GELU(LayerNorm(w_s * W_i state_{i-1} + w_e * Emb_i[token_{i-1}]))
 * for every node of depth i-1, takes the top_k[i] most likely tokens of
 * log_softmax(Head_i state_i) as that node's children, and after n stages keeps
 * the B leaves with the largest summed log-probability.
 *   state     dev [batch, E] weight_dtype      base model's last hidden vector; rows contiguous,
 *                                              16-byte aligned (SPEC_EINVAL otherwise)
 *   last_tok  dev [batch] int32 in [0, V)      token the base model just sampled
 *   top_k     host [n_predict]                 1 <= top_k[i] <= max_top_k[i], <= V
 *   B                                          1 <= B <= prod(top_k) <= SPEC_MAX_LEAVES
 * Outputs (dev, caller-allocated):
 *   cand_tokens [batch, B, n_predict] int32    candidates, most confident first
 *   cand_scores [batch, B] float32             summed log-probability, descending
 *   cand_leaf   [batch, B] int32               leaf index, mixed radix over the ranks
 *                                              (first stage most significant)
 *   dbg        host, may be NULL
 * Ties: larger value first, then smaller token id / leaf index.
 * Errors: SPEC_EINVAL (null, range), SPEC_ESHAPE (exceeds what the model was created for).
 * Calls on one model must not overlap in time: they share the model's workspace. */
spec_status_t spec_draft(spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                         const int32_t* top_k, int32_t B, int32_t* cand_tokens, float* cand_scores,
                         int32_t* cand_leaf, const spec_debug_t* dbg, void* hip_stream);

/* DRAFT with per-sequence speculation settings (Sec. 4.2: speculation is switched off dynamically
 * above a batch size; Sec. 5: the number of candidates is swapped dynamically to the best value for
 * each request).  Sequence q gets its own tree top_k_seq[q][0..n) and keeps B_seq[q] candidates;
 * B_seq[q] = 0 switches speculation off for q (no rows are computed for it).  Sequences do not
 * interact: q's candidates are exactly those of spec_draft on q alone with q's settings.  All
 * sequences share each stage's weight stream (one launch per stage over the ragged row set).
 *   state, last_tok, batch                      as for spec_draft
 *   top_k_seq  host [batch][n_predict]          1 <= top_k_seq[q][i] <= max_top_k[i]; not read where B_seq[q] = 0
 *   B_seq      host [batch]                     0 <= B_seq[q] <= min(B_pad, prod_i top_k_seq[q][i])
 *   B_pad                                       candidate slots per sequence in the outputs, >= 1
 * Outputs (dev, caller-allocated):
 *   cand_tokens [batch, B_pad, n_predict] int32, cand_scores [batch, B_pad] float32, cand_leaf [batch, B_pad]
 *               int32: slots [0, B_seq[q]) as spec_draft writes them (leaf indices in q's own mixed radix);
 *               the slots behind them hold -1 / -inf / -1
 *   n_cand     [batch] int32 = B_seq (the device copy spec_verify_dynamic reads)
 *   dbg        as for spec_draft, with the rows of a stage = those of the active sequences in batch order and
 *              every table of stage i as wide as the widest top_k_seq[.][i] of the call
 * The host arrays are consumed before the call returns.  Unlike spec_draft this call copies a few KB
 * of row maps from host memory to the device on hip_stream (it enqueues kernels and two copies; it may
 * wait for the copy of the call four calls earlier). */
spec_status_t spec_draft_dynamic(spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                                 const int32_t* top_k_seq, const int32_t* B_seq, int32_t B_pad, int32_t* cand_tokens,
                                 float* cand_scores, int32_t* cand_leaf, int32_t* n_cand, const spec_debug_t* dbg,
                                 void* hip_stream);

/* spec_draft for callers that cannot allocate device memory and must not depend on memory
 * somebody allocated for them at run time: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments (no debug outputs), same kernels and the same
 * results as spec_draft, but every intermediate of the call (stage states, projected states,
 * per-part softmax / top-k results, the per-stage tables) lives in a fixed array of
 * SPEC_STATIC_SCRATCH_BYTES that is part of the library's device image, not in the model's
 * workspace.  The call allocates nothing and frees nothing (no hipMalloc / hipFree, no
 * allocating library routine); it only enqueues kernels on hip_stream.
 *   Limit: the workspace of THIS call (it grows with batch * prod(top_k) and with the widths)
 *   must fit the array: SPEC_ESHAPE otherwise, before anything is enqueued.  A 7B-shaped
 *   model with one sequence and the 5/3/2 tree needs 1.2 MB.
 *   The current device must be the model's (SPEC_EINVAL).
 *   Every call on a GPU, from any model and any stream, shares that GPU's array (each GPU the
 *   library runs on holds its own copy until the process ends): calls that overlap in time on
 *   one GPU race, so keep them on one stream or order them with events.  The array keeps the
 *   last call's contents; a call writes every piece before reading it, nothing needs clearing. */
spec_status_t spec_draft_static(spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                                const int32_t* top_k, int32_t B, int32_t* cand_tokens, float* cand_scores,
                                int32_t* cand_leaf, void* hip_stream);

/* VERIFY (Sec. 1, 3.1, 4.1, 5), greedy.
 *   base_logits dev [batch, B, n_predict+1, V] logits_dtype   position p of candidate c is the
 *               base model's output after (last token, cand[c, :p]); position n_predict has
 *               no speculated token and only supplies the bonus token
 *   cand_tokens dev [batch, B, n_predict] int32
 * Outputs (dev, caller-allocated):
 *   greedy      [batch, B, n_predict+1] int32   argmax over V (first maximum); REQUIRED
 *   accept_len  [batch] int32 in [0, n_predict] longest matching prefix of the best candidate
 *   best_cand   [batch] int32 in [0, B)         candidate with the longest prefix (first such)
 *   out_tokens  [batch, n_predict+1] int32      accepted tokens, then the base model's own
 *                                               token at the first position not accepted, then -1
 *   n_out       [batch] int32 = accept_len + 1
 *   accept_all  [batch, B] int32, may be NULL   accepted length of every candidate
 * The caller picks the base model's hidden vector at (best_cand, accept_len) as the next
 * step's state and out_tokens[n_out-1] as its last token. */
spec_status_t spec_verify(const void* base_logits, int32_t logits_dtype, const int32_t* cand_tokens,
                          int32_t batch, int32_t B, int32_t n_predict, int32_t vocab, int32_t* greedy,
                          int32_t* accept_len, int32_t* best_cand, int32_t* out_tokens, int32_t* n_out,
                          int32_t* accept_all, void* hip_stream);

/* VERIFY with per-sequence candidate counts (the counterpart of spec_draft_dynamic; Sec. 4.2, 5).
 *   n_cand dev [batch] int32: sequence q has candidates [0, n_cand[q]) of its B slots; the others are padding
 *   and their base_logits rows are never read.  n_cand[q] = 0 (speculation off): the base model ran an
 *   ordinary decoding step, only base_logits[q, 0, 0, :] is read; accept_len = 0, best_cand = 0,
 *   out_tokens[q] = { its greedy token, -1, .. }, n_out = 1.
 * Everything else as spec_verify; greedy is -1 at positions that were not read, accept_all is 0 for padding. */
spec_status_t spec_verify_dynamic(const void* base_logits, int32_t logits_dtype, const int32_t* cand_tokens,
                                  const int32_t* n_cand, int32_t batch, int32_t B, int32_t n_predict, int32_t vocab,
                                  int32_t* greedy, int32_t* accept_len, int32_t* best_cand, int32_t* out_tokens,
                                  int32_t* n_out, int32_t* accept_all, void* hip_stream);

/* Parity aid: full log-softmax rows of stage `stage`'s head for given states,
 * computed by the same contraction kernels as spec_draft with a store epilogue.
 *   states dev [rows, D] weight_dtype, 16-byte aligned;  logp dev [rows, V] float32;  rows <= max rows of the model. */
spec_status_t spec_head_logp(spec_model_t* m, int32_t stage, const void* states, int32_t rows,
                             float* logp, void* hip_stream);

/* Live timing of the contraction launches (the kernels that bound the step), for
 * roofline reports.  While enabled, spec_draft attaches a pair of HIP events to
 * every contraction launch (they receive that kernel's begin / end time on the
 * caller's stream); nothing else changes.
 *   kernel: 0 = rows<=16 streaming kernel (head_skinny_kernel),
 *           1, 2 = narrow dense kernel head_gemm_kernel<MI,1,8> with MI = 2, 4 (32- / 64-row state blocks),
 *           1000 + 100 * MB + 2 * KT + VT = wide dense kernel head_gemm32_kernel<MB,2,KT,VT>
 *           (32 * MB-row state blocks, per-lane top-k lists of KT entries, VT = 1 with short tiles)
 *   rows, weight_rows, k: the contraction is [rows, k] x [weight_rows, k]^T
 *                  (weight_rows counts head and fused next-projection rows together)
 *   ms: elapsed time between the two events */
typedef struct {
  int32_t kernel, rows, weight_rows, k;
  float ms;
} spec_launch_record_t;

/* capacity > 0: start recording up to `capacity` launches (further launches are not
 * recorded once full, until spec_profile_read empties the recording); capacity == 0: stop and release the events. */
spec_status_t spec_profile_enable(spec_model_t* m, int32_t capacity);

/* Waits for the recorded events, writes up to `cap` records to `out` (host) in launch
 * order, stores their number in *n (host) and clears the recording. */
spec_status_t spec_profile_read(spec_model_t* m, spec_launch_record_t* out, int32_t cap, int32_t* n);

/* Token tree of the candidates (Sec. 3.1: the candidates are evaluated simultaneously with
 * tree attention, which needs every shared prefix once).  Per sequence, with M = B * n_predict:
 *   a node is a distinct prefix cand[c, :p+1]; nodes are numbered in order of first appearance
 *   when the candidates are scanned c = 0..B-1, p = 0..n_predict-1.
 *   node_tok    dev [batch, M] int32  last token of the node's prefix        (-1 past n_nodes)
 *   node_parent dev [batch, M] int32  node of the prefix one shorter; -1 at depth 1 (-1 past n_nodes)
 *   node_depth  dev [batch, M] int32  p + 1                                  (0 past n_nodes)
 *   n_nodes     dev [batch]    int32  number of nodes
 *   cand_node   dev [batch, B, n_predict] int32  node of cand[c, :p+1]
 *   mask        dev [batch, M, M] uint8, may be NULL: mask[i, j] = 1 iff node j is node i or an
 *               ancestor of it; 0 elsewhere (also past n_nodes)
 * cand_tokens dev [batch, B, n_predict] int32 (as written by spec_draft).  All outputs caller-owned.
 * B * n_predict <= 4096.  Asynchronous on hip_stream. */
spec_status_t spec_tree_metadata(const int32_t* cand_tokens, int32_t batch, int32_t B, int32_t n_predict,
                                 int32_t* node_tok, int32_t* node_parent, int32_t* node_depth, int32_t* n_nodes,
                                 int32_t* cand_node, uint8_t* mask, void* hip_stream);

/* Hand-over to the next step without a host round trip (Sec. 3.1: the base model is stage 0 of
 * the draft): the next draft starts from the base model's state vector at the last position
 * whose prediction was kept and from the token predicted there (the bonus token).
 *   hidden      dev [batch, B, n_predict+1, emb_dim] hidden_dtype: base-model states of the
 *               verified positions, aligned with base_logits of spec_verify
 *   best_cand, accept_len, out_tokens: outputs of spec_verify (dev)
 *   next_state  dev [batch, emb_dim] hidden_dtype  = hidden[q, best_cand[q], accept_len[q], :]
 *   next_tok    dev [batch] int32                  = out_tokens[q, accept_len[q]]
 * next_state / next_tok can be passed to the next spec_draft on the same stream. */
spec_status_t spec_advance(const void* hidden, int32_t hidden_dtype, int32_t batch, int32_t B, int32_t n_predict,
                           int32_t emb_dim, const int32_t* best_cand, const int32_t* accept_len,
                           const int32_t* out_tokens, void* next_state, int32_t* next_tok, void* hip_stream);

/* Measurement aid, not a step of the method: one launch of a plain copy kernel that
 * reads `bytes` from src (dev) and writes them to dst (dev; must not overlap src).  Its HBM
 * traffic is known exactly, which calibrates the memory-traffic hardware counters that
 * the roofline reports of the contraction kernels are checked against.
 *   bytes: positive multiple of 16; src, dst 16-byte aligned; asynchronous on hip_stream.
 * SPEC_EINVAL on bad arguments (nothing is launched). */
spec_status_t spec_copy_probe(const void* src, void* dst, int64_t bytes, void* hip_stream);

/* Host-only query (no device, no model, no HIP call): the launch plan the library uses for ONE
 * contraction of the draft (Sec. 3.1: a stage's vocabulary head, with the next stage's state
 * projection riding in the same launch) in the bf16 configuration:
 *   rows    state rows (>= 1);  k  their width (multiple of 64)
 *   n_head  head rows (vocabulary), 0 = no head;  k_top  entries kept per row (1..8; ignored without a head)
 *   n_proj  projection rows, 0 = none (n_head + n_proj >= 1)
 *   n_cu    compute units of the device (256 on MI355X)
 * For checking the planning logic without a GPU and for reading profiles. */
typedef struct {
  int32_t kernel;       /* as spec_launch_record_t.kernel */
  int32_t block_rows;   /* state rows per workgroup */
  int32_t tile_rows;    /* weight rows per workgroup tile */
  int32_t row_blocks;   /* blocks of state rows: row_blocks * block_rows >= rows */
  int32_t ranges;       /* workgroups per row block; each owns a contiguous range of the tiles */
  int32_t tiles;        /* tiles of both weight matrices together */
  int32_t parts;        /* partial (log-sum-exp, top-k) results per row handed to the merge */
  int32_t k_split;      /* workgroups per tile along k (a projection alone), 1 otherwise */
  int32_t workgroups;   /* row_blocks * ranges * k_split */
  int32_t lds_bytes;    /* dynamic LDS per workgroup */
  int32_t proj_apart;   /* 1: spec_draft does not launch this pair as one contraction (its tile list would make
                           the launch one tile longer for a few ranges) but as two, whose plans are those of
                           (n_head, 0) and (0, n_proj); the other fields describe the single launch anyway */
} spec_plan_t;
/* SPEC_EINVAL: arguments out of range; SPEC_ESHAPE: no kernel instance serves the plan (a library bug). */
spec_status_t spec_plan_contraction(int32_t rows, int32_t k, int32_t n_head, int32_t k_top, int32_t n_proj,
                                    int32_t n_cu, spec_plan_t* out);

/* Reads back the mix weights and epsilon the model uses (after defaults were applied). */
spec_status_t spec_model_scalars(const spec_model_t* m, float* state_weight, float* emb_weight,
                                 float* ln_eps);

/* Last error message of the calling thread (static storage, never NULL). */
const char* spec_last_error(void);

/* Library version. */
spec_status_t spec_version(int32_t* major, int32_t* minor);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_DRAFT_H_ */
