// C ABI of libspecdraft (declared in include/spec.h): argument validation,
// model / workspace ownership and the launch sequence of one draft and one
// verify.  All arithmetic lives in the kernels_*.hip files.
#include "../../include/spec.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "spec_internal.h"

using namespace specdraft;

static_assert(SPEC_MAX_TOPK == kMaxTopK, "header and kernels disagree");
static_assert(SPEC_MAX_STAGES == kMaxStages, "header and kernels disagree");
static_assert(SPEC_MAX_LEAVES == kMaxLeaves, "header and kernels disagree");

static thread_local char g_err[512] = "";

static spec_status_t fail(spec_status_t code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
static spec_status_t hip_fail(hipError_t e, const char* what) {
  return fail(SPEC_EHIP, "%s: %s", what, hipGetErrorString(e));
}
#define HIP_TRY(expr)                                  \
  do {                                                 \
    hipError_t e_ = (expr);                            \
    if (e_ != hipSuccess) return hip_fail(e_, #expr);  \
  } while (0)

// Device memory a draft uses beyond its inputs and outputs.  Every buffer is written before it
// is read within one call; nothing has to start at zero.
struct Workspace {
  void* state_in = nullptr;   // bf16: tiled copy of the caller's state (wide dense kernel only)
  void* states = nullptr;     // current stage's states (tiled bf16 / row-major f32)
  float* pz[2] = {nullptr, nullptr};  // projected parent states, ping-pong
  Partials part = {};
  int64_t part_rows_parts = 0;  // capacity in (row, part) slots
  int32_t* tok = nullptr;     // per-stage top-k tables, concatenated
  float* logp = nullptr;
  float* lse = nullptr;
  float* logits = nullptr;    // f32 path and spec_head_logp: materialised rows
  int64_t logits_rows = 0;
};

struct spec_model {
  spec_config_t cfg;
  float w_s, w_e, eps;
  int n_cu;
  int device;
  bool bf16;
  size_t esz;
  // library-owned copies of the contraction weights (bf16: tiled; f32: row-major)
  void* proj[kMaxStages];
  void* head[kMaxStages];
  // borrowed
  const void* emb[kMaxStages];
  const float* gamma[kMaxStages];
  const float* beta[kMaxStages];
  // workspace
  int64_t max_rows;          // largest R_i
  int64_t max_parent_rows;   // largest number of distinct parent states
  int64_t sum_rows, sum_rows_k;
  Workspace ws;
  // per-sequence trees (spec_draft_dynamic): row maps and sequence descriptors are built on the host in
  // one of kDynSlots pinned buffers and copied to dyn_dev on the caller's stream; a slot is reused only
  // after the event recorded behind its copy has completed
  static constexpr int kDynSlots = 4;
  int64_t dyn_ints = 0;
  int32_t* dyn_dev = nullptr;
  int32_t* dyn_host[kDynSlots] = {};
  hipEvent_t dyn_ev[kDynSlots] = {};
  bool dyn_busy[kDynSlots] = {};
  int dyn_next = 0;
  std::vector<void*> owned;
  // live timing of contraction launches
  struct Rec { int kernel, rows, weight_rows, k; };
  std::vector<hipEvent_t> ev;   // 2 per record slot
  std::vector<Rec> rec;
  int prof_cap = 0, prof_n = 0;
};

static void free_model(spec_model* m) {
  if (!m) return;
  for (hipEvent_t e : m->ev) (void)hipEventDestroy(e);
  for (void* p : m->owned)
    if (p) (void)hipFree(p);
  for (int q = 0; q < spec_model::kDynSlots; ++q) {
    if (m->dyn_host[q]) (void)hipHostFree(m->dyn_host[q]);
    if (m->dyn_ev[q]) (void)hipEventDestroy(m->dyn_ev[q]);
  }
  delete m;
}

template <typename T>
static spec_status_t dev_alloc(spec_model* m, T** out, size_t bytes) {
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes ? bytes : 16);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(SPEC_ENOMEM, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
  }
  m->owned.push_back(p);
  *out = static_cast<T*>(p);
  return SPEC_OK;
}

// ---- spec_draft_static: the same draft with its workspace in a static device array ----------
// Each GPU the library runs on holds its own copy of the array until the process ends.  In host code
// the array's name is only a stand-in: its device address is looked up once per device
// (hipGetSymbolAddress) and that pointer is what kernels, copies and fills receive.
static __device__ __align__(256) unsigned char scratch[SPEC_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Address of the CURRENT device's copy of `scratch` (looked up on first use on that device).
static spec_status_t scratch_of_current_device(int* device, unsigned char** out) {
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(SPEC_EINVAL, "device %d is outside the supported range", dev);
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    if (!ptr) return fail(SPEC_EHIP, "hipGetSymbolAddress(scratch) returned a null address");
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
  }
  *device = dev;
  *out = g_scratch_ptr[dev];
  return SPEC_OK;
}

static spec_status_t check_config(const spec_config_t* c) {
  if (!c) return fail(SPEC_EINVAL, "cfg is NULL");
  if (c->n_predict < 1 || c->n_predict > SPEC_MAX_STAGES)
    return fail(SPEC_EINVAL, "n_predict = %d outside [1, %d]", c->n_predict, SPEC_MAX_STAGES);
  if (c->emb_dim < 1 || c->inner_dim < 1 || c->vocab < 1)
    return fail(SPEC_EINVAL, "emb_dim, inner_dim and vocab must be positive");
  if (c->inner_dim > 16384) return fail(SPEC_ESHAPE, "inner_dim = %d exceeds 16384", c->inner_dim);
  if (c->weight_dtype != SPEC_F32 && c->weight_dtype != SPEC_BF16)
    return fail(SPEC_EDTYPE, "weight_dtype = %d is neither SPEC_F32 nor SPEC_BF16", c->weight_dtype);
  if (c->weight_dtype == SPEC_BF16 && (c->emb_dim % 64 || c->inner_dim % 64))
    return fail(SPEC_ESHAPE, "SPEC_BF16 needs emb_dim and inner_dim to be multiples of 64 (got %d, %d)", c->emb_dim,
                c->inner_dim);
  if (c->weight_dtype == SPEC_F32 && (c->inner_dim % 8))
    return fail(SPEC_ESHAPE, "SPEC_F32 needs inner_dim to be a multiple of 8 (got %d)", c->inner_dim);
  if (c->max_batch < 1) return fail(SPEC_EINVAL, "max_batch must be >= 1");
  int64_t leaves = 1, rows = c->max_batch;
  for (int i = 0; i < c->n_predict; ++i) {
    const int k = c->max_top_k[i];
    if (k < 1 || k > SPEC_MAX_TOPK) return fail(SPEC_EINVAL, "max_top_k[%d] = %d outside [1, %d]", i, k, SPEC_MAX_TOPK);
    if (k > c->vocab) return fail(SPEC_EINVAL, "max_top_k[%d] = %d exceeds vocab = %d", i, k, c->vocab);
    leaves *= k;
    if (i + 1 < c->n_predict) rows *= k;
    if (leaves > SPEC_MAX_LEAVES) return fail(SPEC_ESHAPE, "prod(max_top_k) exceeds %d leaves", SPEC_MAX_LEAVES);
    if (rows > (1 << 24)) return fail(SPEC_ESHAPE, "max_batch * prod(max_top_k) is too large");
  }
  if (!std::isfinite(c->state_weight) || !std::isfinite(c->emb_weight) || !std::isfinite(c->ln_eps))
    return fail(SPEC_EINVAL, "state_weight, emb_weight and ln_eps must be finite");
  return SPEC_OK;
}

// capacity (in (row, part) slots) that covers every contraction plan a call may pick:
// the streaming kernel writes one part per workgroup (one per CU), the dense kernel at
// most one per range (<= one per CU, two for blocks of <= 64 rows), the float32 path one per row
static int64_t partial_capacity(int64_t max_rows, int V, int n_cu) {
  (void)V;
  const int64_t cus = n_cu > 0 ? n_cu : 256;
  int64_t cap = 16 * (int64_t)skinny_grid(n_cu);
  if (64 * 2 * cus > cap) cap = 64 * 2 * cus;        // narrow blocks (<= 64 rows): up to two ranges per CU
  if (max_rows * cus > cap) cap = max_rows * cus;
  return cap;
}

extern "C" spec_status_t spec_create(const spec_config_t* cfg, const spec_weights_t* w, void* hip_stream,
                                     spec_model_t** out) {
  spec_status_t st = check_config(cfg);
  if (st != SPEC_OK) return st;
  if (!w || !out) return fail(SPEC_EINVAL, "weights or out is NULL");
  if (!w->proj || !w->emb || !w->head || !w->ln_gamma || !w->ln_beta)
    return fail(SPEC_EINVAL, "a per-stage pointer array of the weights is NULL");
  for (int i = 0; i < cfg->n_predict; ++i)
    if (!w->proj[i] || !w->emb[i] || !w->head[i] || !w->ln_gamma[i] || !w->ln_beta[i])
      return fail(SPEC_EINVAL, "a weight pointer of stage %d is NULL", i);
  // every weight tensor is read with 16-byte loads
  for (int i = 0; i < cfg->n_predict; ++i)
    if ((reinterpret_cast<uintptr_t>(w->proj[i]) | reinterpret_cast<uintptr_t>(w->emb[i]) |
         reinterpret_cast<uintptr_t>(w->head[i]) | reinterpret_cast<uintptr_t>(w->ln_gamma[i]) |
         reinterpret_cast<uintptr_t>(w->ln_beta[i])) & 15)
      return fail(SPEC_EINVAL, "a weight pointer of stage %d is not 16-byte aligned", i);

  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  spec_model* m = new (std::nothrow) spec_model();
  if (!m) return fail(SPEC_ENOMEM, "host allocation failed");
  m->cfg = *cfg;
  const int n = cfg->n_predict, E = cfg->emb_dim, D = cfg->inner_dim, V = cfg->vocab;
  if (cfg->state_weight < 0.f || cfg->emb_weight < 0.f) {
    m->w_s = (float)std::pow(0.5, 1.0 / (2.0 * n));
    m->w_e = (float)std::sqrt(1.0 - std::pow(0.5, 1.0 / n));
  } else {
    m->w_s = cfg->state_weight;
    m->w_e = cfg->emb_weight;
  }
  m->eps = cfg->ln_eps > 0.f ? cfg->ln_eps : 1e-5f;
  m->bf16 = cfg->weight_dtype == SPEC_BF16;
  m->esz = m->bf16 ? 2 : 4;

  int dev = 0;
  hipDeviceProp_t prop;
  hipError_t e = hipGetDevice(&dev);
  if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
  if (e != hipSuccess) {
    free_model(m);
    return hip_fail(e, "hipGetDeviceProperties");
  }
  m->n_cu = prop.multiProcessorCount;
  m->device = dev;
  {
    // set-up for spec_draft_static: this device's address of the static scratch array
    int sdev = -1;
    unsigned char* sptr = nullptr;
    spec_status_t ss = scratch_of_current_device(&sdev, &sptr);
    if (ss != SPEC_OK) {
      free_model(m);
      return ss;
    }
  }

  // rows per stage at the largest call
  int64_t rows = cfg->max_batch, sum_rows = 0, sum_rows_k = 0, max_rows = 0, max_parent = cfg->max_batch;
  for (int i = 0; i < n; ++i) {
    if (rows > max_rows) max_rows = rows;
    if (i + 1 < n && rows > max_parent) max_parent = rows;
    sum_rows += rows;
    sum_rows_k += rows * cfg->max_top_k[i];
    rows *= cfg->max_top_k[i];
  }
  m->max_rows = max_rows;
  m->max_parent_rows = max_parent;
  m->sum_rows = sum_rows;
  m->sum_rows_k = sum_rows_k;

#define TRY_FREE(expr)          \
  do {                          \
    spec_status_t s_ = (expr);  \
    if (s_ != SPEC_OK) {        \
      free_model(m);            \
      return s_;                \
    }                           \
  } while (0)
#define HIP_TRY_FREE(expr)              \
  do {                                  \
    hipError_t e_ = (expr);             \
    if (e_ != hipSuccess) {             \
      free_model(m);                    \
      return hip_fail(e_, #expr);       \
    }                                   \
  } while (0)

  for (int i = 0; i < n; ++i) {
    const int in = i == 0 ? E : D;
    m->emb[i] = w->emb[i];
    m->gamma[i] = w->ln_gamma[i];
    m->beta[i] = w->ln_beta[i];
    // weight-tied stages (the same caller tensor given for several stages) share one copy
    int same_proj = -1, same_head = -1;
    for (int j = 0; j < i; ++j) {
      if (w->proj[j] == w->proj[i] && (j == 0 ? E : D) == in && same_proj < 0) same_proj = j;
      if (w->head[j] == w->head[i] && same_head < 0) same_head = j;
    }
    if (same_proj >= 0) m->proj[i] = m->proj[same_proj];
    if (same_head >= 0) m->head[i] = m->head[same_head];
    if (m->bf16) {
      const size_t pb = (size_t)((D + 15) / 16) * 16 * in * 2, hb = (size_t)((V + 15) / 16) * 16 * D * 2;
      if (same_proj < 0) {
        TRY_FREE(dev_alloc(m, &m->proj[i], pb));
        HIP_TRY_FREE(launch_pack_bf16(w->proj[i], m->proj[i], D, in, true, stream));
      }
      if (same_head < 0) {
        TRY_FREE(dev_alloc(m, &m->head[i], hb));
        HIP_TRY_FREE(launch_pack_bf16(w->head[i], m->head[i], V, D, true, stream));
      }
    } else {
      if (same_proj < 0) {
        TRY_FREE(dev_alloc(m, &m->proj[i], (size_t)D * in * 4));
        HIP_TRY_FREE(hipMemcpyAsync(m->proj[i], w->proj[i], (size_t)D * in * 4, hipMemcpyDeviceToDevice, stream));
      }
      if (same_head < 0) {
        TRY_FREE(dev_alloc(m, &m->head[i], (size_t)V * D * 4));
        HIP_TRY_FREE(hipMemcpyAsync(m->head[i], w->head[i], (size_t)V * D * 4, hipMemcpyDeviceToDevice, stream));
      }
    }
  }

  const int64_t rows16 = (max_rows + 15) / 16 * 16, batch16 = ((int64_t)cfg->max_batch + 15) / 16 * 16;
  TRY_FREE(dev_alloc(m, &m->ws.states, (size_t)rows16 * D * m->esz));
  TRY_FREE(dev_alloc(m, &m->ws.state_in, m->bf16 ? (size_t)batch16 * E * 2 : 16));
  HIP_TRY_FREE(hipMemsetAsync(m->ws.states, 0, (size_t)rows16 * D * m->esz, stream));
  if (m->bf16) HIP_TRY_FREE(hipMemsetAsync(m->ws.state_in, 0, (size_t)batch16 * E * 2, stream));
  // (a projection launched on its own may come as kMaxKSplit partial sums)
  const int64_t pz_rows = (int64_t)kMaxKSplit * max_parent;
  for (int q = 0; q < 2; ++q) TRY_FREE(dev_alloc(m, &m->ws.pz[q], (size_t)pz_rows * D * 4));
  m->ws.part_rows_parts = partial_capacity(max_rows, V, m->n_cu);
  TRY_FREE(dev_alloc(m, &m->ws.part.m, (size_t)m->ws.part_rows_parts * 4));
  TRY_FREE(dev_alloc(m, &m->ws.part.s, (size_t)m->ws.part_rows_parts * 4));
  TRY_FREE(dev_alloc(m, &m->ws.part.val, (size_t)m->ws.part_rows_parts * kMaxTopK * 4));
  TRY_FREE(dev_alloc(m, &m->ws.part.idx, (size_t)m->ws.part_rows_parts * kMaxTopK * 4));
  TRY_FREE(dev_alloc(m, &m->ws.tok, (size_t)sum_rows_k * 4));
  TRY_FREE(dev_alloc(m, &m->ws.logp, (size_t)sum_rows_k * 4));
  TRY_FREE(dev_alloc(m, &m->ws.lse, (size_t)sum_rows * 4));
  // materialised logits: every row for the f32 path, a small window otherwise (spec_head_logp)
  m->ws.logits_rows = m->bf16 ? 0 : max_rows;
  TRY_FREE(dev_alloc(m, &m->ws.logits, (size_t)m->ws.logits_rows * V * 4));

  m->dyn_ints = 2 * sum_rows + (int64_t)cfg->max_batch * (2 * n + 2) + 64;
  TRY_FREE(dev_alloc(m, &m->dyn_dev, (size_t)m->dyn_ints * 4));
  for (int q = 0; q < spec_model::kDynSlots; ++q) {
    HIP_TRY_FREE(hipHostMalloc(reinterpret_cast<void**>(&m->dyn_host[q]), (size_t)m->dyn_ints * 4, hipHostMallocDefault));
    HIP_TRY_FREE(hipEventCreateWithFlags(&m->dyn_ev[q], hipEventDisableTiming));
  }

  HIP_TRY_FREE(hipStreamSynchronize(stream));
#undef TRY_FREE
#undef HIP_TRY_FREE
  *out = m;
  return SPEC_OK;
}

extern "C" void spec_destroy(spec_model_t* m) { free_model(m); }

extern "C" spec_status_t spec_model_scalars(const spec_model_t* m, float* state_weight, float* emb_weight,
                                            float* ln_eps) {
  if (!m) return fail(SPEC_EINVAL, "model is NULL");
  if (state_weight) *state_weight = m->w_s;
  if (emb_weight) *emb_weight = m->w_e;
  if (ln_eps) *ln_eps = m->eps;
  return SPEC_OK;
}

// Reserves a record slot; the launch attaches the slot's two events to the kernel
// dispatch itself, so they carry the kernel's own begin / end timestamps.
static int prof_slot(spec_model* m, int kernel, int rows, int weight_rows, int k) {
  if (m->prof_cap <= 0 || m->prof_n >= m->prof_cap) return -1;
  const int slot = m->prof_n++;
  m->rec[slot] = {kernel, rows, weight_rows, k};
  return slot;
}
#define EV0(slot) ((slot) >= 0 ? m->ev[2 * (slot)] : nullptr)
#define EV1(slot) ((slot) >= 0 ? m->ev[2 * (slot) + 1] : nullptr)

extern "C" spec_status_t spec_profile_enable(spec_model_t* m, int32_t capacity) {
  if (!m) return fail(SPEC_EINVAL, "model is NULL");
  if (capacity < 0 || capacity > (1 << 20)) return fail(SPEC_EINVAL, "capacity = %d out of range", capacity);
  for (hipEvent_t e : m->ev) (void)hipEventDestroy(e);
  m->ev.clear();
  m->rec.clear();
  m->prof_cap = 0;
  m->prof_n = 0;
  for (int i = 0; i < 2 * capacity; ++i) {
    hipEvent_t e;
    HIP_TRY(hipEventCreate(&e));
    m->ev.push_back(e);
  }
  m->rec.resize(capacity);
  m->prof_cap = capacity;
  return SPEC_OK;
}

extern "C" spec_status_t spec_profile_read(spec_model_t* m, spec_launch_record_t* out, int32_t cap, int32_t* n) {
  if (!m || !out || !n) return fail(SPEC_EINVAL, "a required pointer is NULL");
  int w = 0;
  for (int i = 0; i < m->prof_n && w < cap; ++i) {
    HIP_TRY(hipEventSynchronize(m->ev[2 * i + 1]));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, m->ev[2 * i], m->ev[2 * i + 1]));
    out[w].kernel = m->rec[i].kernel;
    out[w].rows = m->rec[i].rows;
    out[w].weight_rows = m->rec[i].weight_rows;
    out[w].k = m->rec[i].k;
    out[w].ms = ms;
    ++w;
  }
  *n = w;
  m->prof_n = 0;
  return SPEC_OK;
}

extern "C" spec_status_t spec_plan_contraction(int32_t rows, int32_t k, int32_t n_head, int32_t k_top, int32_t n_proj,
                                               int32_t n_cu, spec_plan_t* out) {
  if (!out) return fail(SPEC_EINVAL, "out is NULL");
  if (rows < 1 || k < 64 || k % 64) return fail(SPEC_EINVAL, "rows = %d, k = %d: need rows >= 1, k a positive multiple of 64", rows, k);
  if (n_head < 0 || n_proj < 0 || n_head + (int64_t)n_proj < 1)
    return fail(SPEC_EINVAL, "n_head = %d, n_proj = %d: need at least one weight row", n_head, n_proj);
  if (n_head > 0 && (k_top < 1 || k_top > kMaxTopK)) return fail(SPEC_EINVAL, "k_top = %d outside [1, %d]", k_top, kMaxTopK);
  if (n_cu < 1) return fail(SPEC_EINVAL, "n_cu = %d must be >= 1", n_cu);
  memset(out, 0, sizeof(*out));
  const int kt = k / 32;
  if (skinny_fits(rows, kt)) {
    out->kernel = 0;
    out->block_rows = 16;
    out->tile_rows = 16;
    out->row_blocks = 1;
    out->ranges = skinny_grid(n_cu);
    out->tiles = (n_head + 15) / 16 + (n_proj + 15) / 16;
    out->parts = skinny_grid(n_cu);
    out->k_split = 1;
    out->workgroups = skinny_grid(n_cu);
    out->lds_bytes = (int32_t)skinny_lds_bytes(rows, kt);
    return SPEC_OK;
  }
  GemmPlan pl = plan_gemm(rows, n_head > 0 ? k_top : 0, n_head, n_proj, kt, n_cu);
  HeadJob job;
  memset(&job, 0, sizeof(job));
  job.kt = kt;
  job.R = rows;
  job.k_top = n_head > 0 ? k_top : 0;
  job.n_head = n_head;
  job.vt_head = (n_head + 15) / 16;
  job.n_proj = n_proj;
  job.vt_proj = (n_proj + 15) / 16;
  job.ld_head = n_head;
  job.ld_proj = n_proj;
  job.proj_part_stride = (int64_t)rows * n_proj;
  size_t lds = 0;
  if (launch_head_gemm(job, pl, nullptr, nullptr, nullptr, &lds) != hipSuccess)
    return fail(SPEC_ESHAPE, "no kernel instance for %d-row blocks, %d weight rows per wave, top-k lists of %d, tiles of %d",
                16 * pl.mi, 16 * pl.ni, pl.kcap, 16 * pl.ts);
  out->kernel = pl.ni == 1 ? (pl.mi == 2 ? 1 : 2) : 1000 + 50 * pl.mi + 2 * pl.kcap + (pl.ts != 16 ? 1 : 0);
  out->block_rows = 16 * pl.mi;
  out->tile_rows = 16 * pl.ts;
  out->row_blocks = pl.m_tiles;
  out->ranges = pl.n_ranges;
  out->tiles = ((n_head + 15) / 16 + pl.ts - 1) / pl.ts + ((n_proj + 15) / 16 + pl.ts - 1) / pl.ts;
  out->parts = pl.nparts;
  out->k_split = pl.ksplit;
  out->workgroups = pl.m_tiles * pl.n_ranges * pl.ksplit;
  out->lds_bytes = (int32_t)lds;
  out->proj_apart = plan_projection_apart(rows, job.k_top, n_head, n_proj, kt, n_cu) ? 1 : 0;
  return SPEC_OK;
}

extern "C" spec_status_t spec_copy_probe(const void* src, void* dst, int64_t bytes, void* hip_stream) {
  if (!src || !dst) return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (bytes <= 0 || bytes % 16) return fail(SPEC_EINVAL, "bytes = %lld must be a positive multiple of 16", (long long)bytes);
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15)
    return fail(SPEC_EINVAL, "src and dst must be 16-byte aligned");
  HIP_TRY(launch_copy_probe(src, dst, bytes / 16, static_cast<hipStream_t>(hip_stream)));
  return SPEC_OK;
}

// One contraction of R state rows against head[stage] (top-k partials, or raw
// logits into out_head) and, if proj_stage >= 0, against proj[proj_stage]
// (stored to out_proj).  Returns the number of parts per row it produced.
static HeadJob make_head_job(const spec_model* m, const Workspace& ws, int stage, int proj_stage, const void* b_src, bool b_rowmajor,
                             int b_ld, int R, int k_top, float* out_head, float* out_proj) {
  const int D = m->cfg.inner_dim, V = m->cfg.vocab;
  HeadJob job;
  memset(&job, 0, sizeof(job));
  job.kt = b_ld / 32;
  job.b_src = b_src;
  job.b_rowmajor = b_rowmajor ? 1 : 0;
  job.b_ld = b_ld;
  job.R = R;
  job.k_top = k_top;
  job.part = ws.part;
  job.out_head = out_head;
  job.ld_head = V;
  job.out_proj = out_proj;
  job.ld_proj = D;
  if (stage >= 0) {
    job.w_head = m->head[stage];
    job.vt_head = (V + 15) / 16;
    job.n_head = V;
  }
  if (proj_stage >= 0) {
    job.w_proj = m->proj[proj_stage];
    job.vt_proj = (D + 15) / 16;
    job.n_proj = D;
  }
  return job;
}

static spec_status_t run_contraction(spec_model* m, const Workspace& ws, int stage, int proj_stage, const void* b_src, bool b_rowmajor,
                                     int b_ld, int R, int k_top, float* out_head, float* out_proj, int* nparts,
                                     hipStream_t st, int* proj_parts = nullptr, const FoldJob* fold = nullptr) {
  if (proj_parts) *proj_parts = 1;
  HeadJob job = make_head_job(m, ws, stage, proj_stage, b_src, b_rowmajor, b_ld, R, k_top, out_head, out_proj);
  const int K = b_ld;
  if (fold && !skinny_fits(R, job.kt)) return fail(SPEC_ESHAPE, "internal: folded stage on a contraction of %d rows", R);
  if (fold) job.fold = *fold;
  if (skinny_fits(R, job.kt)) {
    job.nparts = skinny_grid(m->n_cu);
    *nparts = job.nparts;
    const int slot = prof_slot(m, 0, R, job.n_head + job.n_proj, K);
    HIP_TRY(launch_head_skinny(job, m->n_cu, st, EV0(slot), EV1(slot)));
    return SPEC_OK;
  }
  GemmPlan pl = plan_gemm(R, k_top, job.n_head, job.n_proj, job.kt, m->n_cu);
  // the wide kernel wants tiled states; the narrow one gathers row-major rows itself
  if (b_rowmajor && pl.ni != 1) {
    HIP_TRY(launch_pack_bf16(b_src, ws.state_in, R, K, false, st));
    job.b_src = ws.state_in;
    job.b_rowmajor = 0;
  }
  if (pl.ksplit > 1) {
    if (!proj_parts) pl.ksplit = 1;  // the caller reads out_proj as it is
    else job.proj_part_stride = (int64_t)R * job.ld_proj;
  }
  if (proj_parts) *proj_parts = pl.ksplit;
  job.nparts = pl.nparts > 0 ? pl.nparts : 1;
  *nparts = job.nparts;
  if (stage >= 0 && !out_head && (int64_t)R * job.nparts > ws.part_rows_parts)
    return fail(SPEC_ESHAPE, "internal: partial workspace too small (%d rows x %d parts)", R, job.nparts);
  const int slot = prof_slot(m, pl.ni == 1 ? (pl.mi == 2 ? 1 : 2) : 1000 + 50 * pl.mi + 2 * pl.kcap + (pl.ts != 16 ? 1 : 0), R, job.n_head + job.n_proj, K);
  HIP_TRY(launch_head_gemm(job, pl, st, EV0(slot), EV1(slot)));
  return SPEC_OK;
}

// Per-sequence trees of one call (spec_draft_dynamic): rows and table widths per stage and the
// device copies of the row maps / sequence descriptors the stage and tree kernels read.
struct DynPlan {
  int64_t R[kMaxStages];             // rows per stage over all sequences
  int kw[kMaxStages];                // widest branching per stage = table width and top-k of the head launch
  const int32_t* parent[kMaxStages]; // dev, [R_i]
  const int32_t* rank[kMaxStages];   // dev, [R_i]
  const int32_t* seq_desc;           // dev, [batch][2 n + 1]
  int B_pad;
};

// Host-side checks of a draft call's arguments (no HIP call).
static spec_status_t check_draft(const spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                                 const int32_t* top_k, int32_t B, const int32_t* cand_tokens, const float* cand_scores,
                                 const int32_t* cand_leaf) {
  if (!m) return fail(SPEC_EINVAL, "model is NULL");
  if (!state || !last_tok || !top_k || !cand_tokens || !cand_scores || !cand_leaf)
    return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (batch < 1) return fail(SPEC_EINVAL, "batch = %d must be >= 1", batch);
  if (reinterpret_cast<uintptr_t>(state) & 15) return fail(SPEC_EINVAL, "state must be 16-byte aligned");
  if (batch > m->cfg.max_batch) return fail(SPEC_ESHAPE, "batch = %d exceeds max_batch = %d", batch, m->cfg.max_batch);
  int64_t L = 1;
  for (int i = 0; i < m->cfg.n_predict; ++i) {
    if (top_k[i] < 1) return fail(SPEC_EINVAL, "top_k[%d] = %d must be >= 1", i, top_k[i]);
    if (top_k[i] > m->cfg.max_top_k[i])
      return fail(SPEC_ESHAPE, "top_k[%d] = %d exceeds max_top_k[%d] = %d", i, top_k[i], i, m->cfg.max_top_k[i]);
    L *= top_k[i];
  }
  if (B < 1 || B > L) return fail(SPEC_EINVAL, "B = %d outside [1, prod(top_k) = %lld]", B, (long long)L);
  return SPEC_OK;
}

// One draft (arguments already checked) with the workspace `ws`: the model's own, or one carved
// from the static scratch array.
static spec_status_t draft_impl(spec_model_t* m, const Workspace& ws, const void* state,
                                const int32_t* last_tok, int32_t batch, const int32_t* top_k, int32_t B,
                                int32_t* cand_tokens, float* cand_scores, int32_t* cand_leaf, const spec_debug_t* dbg,
                                void* hip_stream, const DynPlan* dyn = nullptr) {
  // dyn != nullptr: per-sequence trees; top_k then holds the widest branching per stage (dyn->kw) and B is unused
  const int n = m->cfg.n_predict, E = m->cfg.emb_dim, D = m->cfg.inner_dim, V = m->cfg.vocab;
  int64_t L = 1;
  for (int i = 0; i < n; ++i) L *= top_k[i];
  if (dyn) L = 1;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);

  // rows and table offsets per stage
  int64_t R[kMaxStages], off[kMaxStages], row_off[kMaxStages];
  {
    int64_t r = batch, o = 0, ro = 0;
    for (int i = 0; i < n; ++i) {
      if (dyn) r = dyn->R[i];
      R[i] = r;
      off[i] = o;
      row_off[i] = ro;
      o += r * top_k[i];
      ro += r;
      r *= top_k[i];
    }
  }

  auto stage_job = [&](int i, int nparts) {
    StageJob sj;
    memset(&sj, 0, sizeof(sj));
    sj.stage = i;
    sj.R = (int)R[i];
    sj.k_prev = i == 0 ? 1 : top_k[i - 1];
    sj.xcd_rows = (m->bf16 && R[i] > 16) ? 1 : 0;   // more than one tile of packed states
    sj.D = D;
    sj.bf16 = m->bf16 ? 1 : 0;
    sj.part = ws.part;
    sj.nparts = nparts;
    sj.V = V;
    if (i > 0) {
      sj.prev_tok = ws.tok + off[i - 1];
      sj.prev_logp = ws.logp + off[i - 1];
      sj.prev_lse = ws.lse + row_off[i - 1];
    }
    sj.last_tok = last_tok;
    sj.pz = ws.pz[i & 1];
    sj.emb = m->emb[i];
    sj.gamma = m->gamma[i];
    sj.beta = m->beta[i];
    sj.w_s = m->w_s;
    sj.w_e = m->w_e;
    sj.eps = m->eps;
    sj.state_out = ws.states;
    sj.state_dbg = (dbg && dbg->stage_state)
                       ? static_cast<void*>(static_cast<char*>(dbg->stage_state) + (size_t)row_off[i] * D * m->esz)
                       : nullptr;
    if (dyn) {
      sj.row_parent = dyn->parent[i];
      sj.row_rank = dyn->rank[i];
    }
    return sj;
  };
  auto tree_job = [&](int nparts) {
    TreeJob tj;
    memset(&tj, 0, sizeof(tj));
    tj.batch = batch;
    tj.n = n;
    tj.B = B;
    tj.B_pad = dyn ? dyn->B_pad : B;
    tj.seq_desc = dyn ? dyn->seq_desc : nullptr;
    tj.L = (int)L;
    for (int i = 0; i < n; ++i) {
      tj.kstride[i] = top_k[i];
      tj.top_k[i] = top_k[i];
      tj.off[i] = off[i];
      tj.row_off[i] = row_off[i];
    }
    for (int i = n; i < kMaxStages; ++i) tj.top_k[i] = 1;
    tj.part = ws.part;
    tj.nparts = nparts;
    tj.tok = ws.tok;
    tj.logp = ws.logp;
    tj.lse = ws.lse;
    tj.cand_tokens = cand_tokens;
    tj.cand_scores = cand_scores;
    tj.cand_leaf = cand_leaf;
    return tj;
  };

  {
    int nparts = 1, pz0_parts = 1;
    const bool any_rows = R[0] > 0;   // (per-sequence trees: every sequence may have speculation switched off)
    // projection of the base model's state for stage 1
    if (!any_rows) {
    } else if (m->bf16) {
      spec_status_t s = run_contraction(m, ws, -1, 0, state, true, E, batch, 0, nullptr, ws.pz[0], &nparts, st, &pz0_parts);
      if (s != SPEC_OK) return s;
    } else {
      HIP_TRY(launch_gemm_f32(static_cast<const float*>(state), E, static_cast<const float*>(m->proj[0]), E, ws.pz[0],
                              D, batch, D, E, st));
    }

    int pz_parts = pz0_parts;                 // parts of the projection the current stage reads
    int64_t pz_part_stride = (int64_t)batch * D;
    for (int i = 0; any_rows && i < n; ++i) {
      StageJob sj = stage_job(i, nparts);
      sj.pz_parts = pz_parts;
      sj.pz_part_stride = pz_part_stride;
      pz_parts = 1;
      // First stage of one or two sequences: its rows (token = the last sampled one, no merge) are
      // computed inside the head's streaming kernel instead of by a launch of their own.
      FoldJob fold;
      memset(&fold, 0, sizeof(fold));
      const bool folded = i == 0 && m->bf16 && !dbg && !dyn && skinny_fits((int)R[0], D / 32) && (int)R[0] <= skinny_fold_rows(D);
      if (folded) {
        fold.enabled = 1;
        fold.D = D; fold.V = V;
        fold.pz = sj.pz; fold.pz_parts = sj.pz_parts > 0 ? sj.pz_parts : 1; fold.pz_part_stride = sj.pz_part_stride;
        fold.tok = last_tok;
        fold.emb = sj.emb; fold.gamma = sj.gamma; fold.beta = sj.beta;
        fold.w_s = sj.w_s; fold.w_e = sj.w_e; fold.eps = sj.eps;
      } else {
        HIP_TRY(launch_stage(sj, st));
      }
      const int proj_next = i + 1 < n ? i + 1 : -1;
      if (m->bf16 && proj_next >= 0 && !skinny_fits((int)R[i], D / 32) &&
          plan_projection_apart((int)R[i], top_k[i], V, D, D / 32, m->n_cu)) {
        // the head in one even round of tiles, then the next projection on its own, split along K
        spec_status_t s = run_contraction(m, ws, i, -1, ws.states, false, D, (int)R[i], top_k[i], nullptr, nullptr,
                                          &nparts, st);
        if (s != SPEC_OK) return s;
        int np_unused = 0;
        s = run_contraction(m, ws, -1, proj_next, ws.states, false, D, (int)R[i], 0, nullptr, ws.pz[(i + 1) & 1],
                            &np_unused, st, &pz_parts);
        if (s != SPEC_OK) return s;
        pz_part_stride = R[i] * D;
      } else if (m->bf16) {
        spec_status_t s = run_contraction(m, ws, i, proj_next, ws.states, false, D, (int)R[i], top_k[i], nullptr,
                                          ws.pz[(i + 1) & 1], &nparts, st, nullptr, folded ? &fold : nullptr);
        if (s != SPEC_OK) return s;
      } else {
        const float* sf = static_cast<const float*>(ws.states);
        HIP_TRY(launch_gemm_f32(sf, D, static_cast<const float*>(m->head[i]), D, ws.logits, V, (int)R[i], V, D, st));
        HIP_TRY(launch_row_topk_f32(ws.logits, V, (int)R[i], V, top_k[i], ws.part, st));
        nparts = 1;
        if (proj_next >= 0)
          HIP_TRY(launch_gemm_f32(sf, D, static_cast<const float*>(m->proj[proj_next]), D, ws.pz[(i + 1) & 1], D,
                                  (int)R[i], D, D, st));
      }
    }
    HIP_TRY(launch_tree(tree_job(nparts), st));
  }

  if (dbg) {
    const int64_t nk = off[n - 1] + R[n - 1] * top_k[n - 1], nr = row_off[n - 1] + R[n - 1];
    if (dbg->topk_tok) HIP_TRY(hipMemcpyAsync(dbg->topk_tok, ws.tok, (size_t)nk * 4, hipMemcpyDeviceToDevice, st));
    if (dbg->topk_logp) HIP_TRY(hipMemcpyAsync(dbg->topk_logp, ws.logp, (size_t)nk * 4, hipMemcpyDeviceToDevice, st));
    if (dbg->row_lse) HIP_TRY(hipMemcpyAsync(dbg->row_lse, ws.lse, (size_t)nr * 4, hipMemcpyDeviceToDevice, st));
  }
  return SPEC_OK;
}

extern "C" spec_status_t spec_draft(spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                                    const int32_t* top_k, int32_t B, int32_t* cand_tokens, float* cand_scores,
                                    int32_t* cand_leaf, const spec_debug_t* dbg, void* hip_stream) {
  spec_status_t s = check_draft(m, state, last_tok, batch, top_k, B, cand_tokens, cand_scores, cand_leaf);
  if (s != SPEC_OK) return s;
  return draft_impl(m, m->ws, state, last_tok, batch, top_k, B, cand_tokens, cand_scores, cand_leaf, dbg,
                    hip_stream);
}

// ---- spec_draft_dynamic: own tree and candidate count per sequence -------------------------------
extern "C" spec_status_t spec_draft_dynamic(spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                                            const int32_t* top_k_seq, const int32_t* B_seq, int32_t B_pad,
                                            int32_t* cand_tokens, float* cand_scores, int32_t* cand_leaf,
                                            int32_t* n_cand, const spec_debug_t* dbg, void* hip_stream) {
  if (!m) return fail(SPEC_EINVAL, "model is NULL");
  if (!state || !last_tok || !top_k_seq || !B_seq || !cand_tokens || !cand_scores || !cand_leaf || !n_cand)
    return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (batch < 1) return fail(SPEC_EINVAL, "batch = %d must be >= 1", batch);
  if (reinterpret_cast<uintptr_t>(state) & 15) return fail(SPEC_EINVAL, "state must be 16-byte aligned");
  if (batch > m->cfg.max_batch) return fail(SPEC_ESHAPE, "batch = %d exceeds max_batch = %d", batch, m->cfg.max_batch);
  if (B_pad < 1) return fail(SPEC_EINVAL, "B_pad = %d must be >= 1", B_pad);
  const int n = m->cfg.n_predict;
  DynPlan dp;
  memset(&dp, 0, sizeof(dp));
  dp.B_pad = B_pad;
  int kw[kMaxStages];
  for (int i = 0; i < n; ++i) kw[i] = 1;
  for (int q = 0; q < batch; ++q) {
    const int Bq = B_seq[q];
    if (Bq < 0 || Bq > B_pad) return fail(SPEC_EINVAL, "B_seq[%d] = %d outside [0, B_pad = %d]", q, Bq, B_pad);
    if (Bq == 0) continue;   // speculation off: the sequence's top_k entries are not read
    int64_t L = 1;
    for (int i = 0; i < n; ++i) {
      const int k = top_k_seq[(int64_t)q * n + i];
      if (k < 1) return fail(SPEC_EINVAL, "top_k_seq[%d][%d] = %d must be >= 1", q, i, k);
      if (k > m->cfg.max_top_k[i])
        return fail(SPEC_ESHAPE, "top_k_seq[%d][%d] = %d exceeds max_top_k[%d] = %d", q, i, k, i, m->cfg.max_top_k[i]);
      if (k > kw[i]) kw[i] = k;
      dp.R[i] += L;
      L *= k;
    }
    if (Bq > L) return fail(SPEC_EINVAL, "B_seq[%d] = %d exceeds the %lld leaves of its tree", q, Bq, (long long)L);
  }
  int64_t ints = (int64_t)batch * (2 * n + 1);
  for (int i = 0; i < n; ++i) ints += 2 * dp.R[i];
  if (ints > m->dyn_ints) return fail(SPEC_ESHAPE, "internal: row maps of %lld words exceed the model's %lld", (long long)ints, (long long)m->dyn_ints);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);

  // a free pinned slot (the copy out of it may still be pending on the caller's stream)
  const int slot = m->dyn_next;
  m->dyn_next = (slot + 1) % spec_model::kDynSlots;
  if (m->dyn_busy[slot]) HIP_TRY(hipEventSynchronize(m->dyn_ev[slot]));
  int32_t* h = m->dyn_host[slot];
  // layout: per stage parent[R_i], rank[R_i]; then the sequence descriptors; then B_seq (for n_cand)
  int64_t at = 0, p_at[kMaxStages], r_at[kMaxStages];
  for (int i = 0; i < n; ++i) {
    p_at[i] = at;
    at += dp.R[i];
    r_at[i] = at;
    at += dp.R[i];
  }
  const int64_t d_at = at;
  int64_t row0[kMaxStages];
  for (int i = 0; i < n; ++i) row0[i] = 0;
  for (int q = 0; q < batch; ++q) {
    int32_t* d = h + d_at + (int64_t)q * (2 * n + 1);
    const int Bq = B_seq[q];
    d[2 * n] = Bq;
    int64_t cnt = 1;
    for (int i = 0; i < n; ++i) {
      const int k = Bq > 0 ? top_k_seq[(int64_t)q * n + i] : 1;
      d[i] = k;
      d[n + i] = (int32_t)row0[i];
      if (Bq > 0) {
        const int k_prev = i == 0 ? 1 : top_k_seq[(int64_t)q * n + i - 1];
        for (int64_t l = 0; l < cnt; ++l) {
          // stage 0 hangs under the sequence itself; later rows under row l / k_prev of the previous stage
          h[p_at[i] + row0[i] + l] = i == 0 ? q : (int32_t)(row0[i - 1] - cnt / k_prev + l / k_prev);
          h[r_at[i] + row0[i] + l] = i == 0 ? 0 : (int32_t)(l % k_prev);
        }
        row0[i] += cnt;
        cnt *= k;
      }
    }
  }
  // n_cand for the verify side: the B_seq values, from the same pinned slot
  int32_t* hb = h + ints;
  if (ints + batch > m->dyn_ints) return fail(SPEC_ESHAPE, "internal: row maps exceed the model's buffer");
  for (int q = 0; q < batch; ++q) hb[q] = B_seq[q];
  HIP_TRY(hipMemcpyAsync(m->dyn_dev, h, (size_t)ints * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(hipMemcpyAsync(n_cand, hb, (size_t)batch * 4, hipMemcpyHostToDevice, st));
  HIP_TRY(hipEventRecord(m->dyn_ev[slot], st));
  m->dyn_busy[slot] = true;
  for (int i = 0; i < n; ++i) {
    dp.kw[i] = kw[i];
    dp.parent[i] = m->dyn_dev + p_at[i];
    dp.rank[i] = m->dyn_dev + r_at[i];
  }
  dp.seq_desc = m->dyn_dev + d_at;
  return draft_impl(m, m->ws, state, last_tok, batch, kw, 1, cand_tokens, cand_scores, cand_leaf, dbg, hip_stream,
                    &dp);
}

// ---- spec_draft_static: the same draft, its workspace carved from the static device array ----
// Lays the workspace of one call (batch, top_k) out inside [base, base + SPEC_STATIC_SCRATCH_BYTES):
// sized for THIS call (not for the model's maxima), every piece on a 256-byte boundary.
static spec_status_t carve_static(const spec_model* m, unsigned char* base, int batch, const int32_t* top_k,
                                  Workspace* ws) {
  const int n = m->cfg.n_predict, E = m->cfg.emb_dim, D = m->cfg.inner_dim, V = m->cfg.vocab;
  int64_t rows = batch, sum_rows = 0, sum_rows_k = 0, max_rows = 0, max_parent = batch;
  for (int i = 0; i < n; ++i) {
    if (rows > max_rows) max_rows = rows;
    if (i + 1 < n && rows > max_parent) max_parent = rows;
    sum_rows += rows;
    sum_rows_k += rows * top_k[i];
    rows *= top_k[i];
  }
  size_t used = 0;
  bool fits = true;
  auto take = [&](size_t bytes) -> unsigned char* {
    unsigned char* p = base + used;
    used += (bytes + 255) & ~(size_t)255;
    if (used > (size_t)SPEC_STATIC_SCRATCH_BYTES) fits = false;
    return p;
  };
  const int64_t rows16 = (max_rows + 15) / 16 * 16, batch16 = ((int64_t)batch + 15) / 16 * 16;
  const int64_t pz_rows = (int64_t)kMaxKSplit * max_parent;
  // parts per row: one per workgroup of the streaming kernel when every stage has at most 16 rows,
  // else what the dense plans may produce
  const int64_t cap = max_rows <= 16 && m->bf16 ? 16 * (int64_t)skinny_grid(m->n_cu) : partial_capacity(max_rows, V, m->n_cu);
  ws->states = take((size_t)rows16 * D * m->esz);
  ws->state_in = take(m->bf16 ? (size_t)batch16 * E * 2 : 16);
  for (int q = 0; q < 2; ++q) ws->pz[q] = reinterpret_cast<float*>(take((size_t)pz_rows * D * 4));
  ws->part_rows_parts = cap;
  ws->part.m = reinterpret_cast<float*>(take((size_t)cap * 4));
  ws->part.s = reinterpret_cast<float*>(take((size_t)cap * 4));
  ws->part.val = reinterpret_cast<float*>(take((size_t)cap * kMaxTopK * 4));
  ws->part.idx = reinterpret_cast<int32_t*>(take((size_t)cap * kMaxTopK * 4));
  ws->tok = reinterpret_cast<int32_t*>(take((size_t)sum_rows_k * 4));
  ws->logp = reinterpret_cast<float*>(take((size_t)sum_rows_k * 4));
  ws->lse = reinterpret_cast<float*>(take((size_t)sum_rows * 4));
  ws->logits_rows = m->bf16 ? 0 : max_rows;
  ws->logits = reinterpret_cast<float*>(take((size_t)ws->logits_rows * V * 4));
  if (!fits)
    return fail(SPEC_ESHAPE, "spec_draft_static: this call needs %zu bytes of workspace, the static array holds %d "
                             "(use spec_draft for larger batches or trees)", used, SPEC_STATIC_SCRATCH_BYTES);
  return SPEC_OK;
}

extern "C" spec_status_t spec_draft_static(spec_model_t* m, const void* state, const int32_t* last_tok, int32_t batch,
                                           const int32_t* top_k, int32_t B, int32_t* cand_tokens, float* cand_scores,
                                           int32_t* cand_leaf, void* hip_stream) {
  spec_status_t s = check_draft(m, state, last_tok, batch, top_k, B, cand_tokens, cand_scores, cand_leaf);
  if (s != SPEC_OK) return s;
  Workspace ws;
  int dev = -1;
  unsigned char* base = nullptr;
  s = scratch_of_current_device(&dev, &base);
  if (s != SPEC_OK) return s;
  if (dev != m->device)
    return fail(SPEC_EINVAL, "the model lives on device %d, the current device is %d", m->device, dev);
  s = carve_static(m, base, batch, top_k, &ws);
  if (s != SPEC_OK) return s;
  return draft_impl(m, ws, state, last_tok, batch, top_k, B, cand_tokens, cand_scores, cand_leaf, nullptr,
                    hip_stream);
}

extern "C" spec_status_t spec_head_logp(spec_model_t* m, int32_t stage, const void* states, int32_t rows, float* logp,
                                        void* hip_stream) {
  if (!m) return fail(SPEC_EINVAL, "model is NULL");
  if (!states || !logp) return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (stage < 0 || stage >= m->cfg.n_predict) return fail(SPEC_EINVAL, "stage = %d out of range", stage);
  if (reinterpret_cast<uintptr_t>(states) & 15) return fail(SPEC_EINVAL, "states must be 16-byte aligned");
  if (rows < 1 || rows > m->max_rows) return fail(SPEC_ESHAPE, "rows = %d outside [1, %lld]", rows, (long long)m->max_rows);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int D = m->cfg.inner_dim, V = m->cfg.vocab;
  if (m->bf16) {
    int nparts = 0;
    if (skinny_fits(rows, D / 32)) {
      spec_status_t s = run_contraction(m, m->ws, stage, -1, states, true, D, rows, 0, logp, nullptr, &nparts, st);
      if (s != SPEC_OK) return s;
    } else {
      // tile the rows into the model's state buffer, then contract with the store epilogue
      HIP_TRY(launch_pack_bf16(states, m->ws.states, rows, D, false, st));
      spec_status_t s = run_contraction(m, m->ws, stage, -1, m->ws.states, false, D, rows, 0, logp, nullptr, &nparts, st);
      if (s != SPEC_OK) return s;
    }
  } else {
    HIP_TRY(launch_gemm_f32(static_cast<const float*>(states), D, static_cast<const float*>(m->head[stage]), D, logp, V,
                            rows, V, D, st));
  }
  HIP_TRY(launch_row_log_softmax(logp, logp, V, rows, V, st));
  return SPEC_OK;
}

static spec_status_t verify_impl(const void* base_logits, int32_t logits_dtype, const int32_t* cand_tokens,
                                 const int32_t* n_cand, int32_t batch, int32_t B, int32_t n_predict, int32_t vocab,
                                 int32_t* greedy, int32_t* accept_len, int32_t* best_cand, int32_t* out_tokens,
                                 int32_t* n_out, int32_t* accept_all, void* hip_stream) {
  if (!base_logits || !cand_tokens || !greedy || !accept_len || !best_cand || !out_tokens || !n_out)
    return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (logits_dtype != SPEC_F32 && logits_dtype != SPEC_BF16)
    return fail(SPEC_EDTYPE, "logits_dtype = %d is neither SPEC_F32 nor SPEC_BF16", logits_dtype);
  if (batch < 1 || B < 1 || vocab < 1) return fail(SPEC_EINVAL, "batch, B and vocab must be >= 1");
  if (n_predict < 1 || n_predict > SPEC_MAX_STAGES)
    return fail(SPEC_EINVAL, "n_predict = %d outside [1, %d]", n_predict, SPEC_MAX_STAGES);
  const int64_t rows = (int64_t)batch * B * (n_predict + 1);
  if (rows > 0x7fffffffLL) return fail(SPEC_ESHAPE, "batch * B * (n_predict + 1) is too large");
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  HIP_TRY(launch_argmax_rows(base_logits, logits_dtype == SPEC_BF16, rows, vocab, B, n_predict + 1, n_cand, greedy, st));
  HIP_TRY(launch_accept(greedy, cand_tokens, n_cand, batch, B, n_predict, accept_len, best_cand, out_tokens, n_out,
                        accept_all, st));
  return SPEC_OK;
}

extern "C" spec_status_t spec_verify(const void* base_logits, int32_t logits_dtype, const int32_t* cand_tokens,
                                     int32_t batch, int32_t B, int32_t n_predict, int32_t vocab, int32_t* greedy,
                                     int32_t* accept_len, int32_t* best_cand, int32_t* out_tokens, int32_t* n_out,
                                     int32_t* accept_all, void* hip_stream) {
  return verify_impl(base_logits, logits_dtype, cand_tokens, nullptr, batch, B, n_predict, vocab, greedy, accept_len,
                     best_cand, out_tokens, n_out, accept_all, hip_stream);
}

extern "C" spec_status_t spec_verify_dynamic(const void* base_logits, int32_t logits_dtype, const int32_t* cand_tokens,
                                             const int32_t* n_cand, int32_t batch, int32_t B, int32_t n_predict,
                                             int32_t vocab, int32_t* greedy, int32_t* accept_len, int32_t* best_cand,
                                             int32_t* out_tokens, int32_t* n_out, int32_t* accept_all,
                                             void* hip_stream) {
  if (!n_cand) return fail(SPEC_EINVAL, "n_cand is NULL");
  return verify_impl(base_logits, logits_dtype, cand_tokens, n_cand, batch, B, n_predict, vocab, greedy, accept_len,
                     best_cand, out_tokens, n_out, accept_all, hip_stream);
}

extern "C" spec_status_t spec_tree_metadata(const int32_t* cand_tokens, int32_t batch, int32_t B, int32_t n_predict,
                                            int32_t* node_tok, int32_t* node_parent, int32_t* node_depth,
                                            int32_t* n_nodes, int32_t* cand_node, uint8_t* mask, void* hip_stream) {
  if (!cand_tokens || !node_tok || !node_parent || !node_depth || !n_nodes || !cand_node)
    return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (batch < 1 || B < 1) return fail(SPEC_EINVAL, "batch and B must be >= 1");
  if (n_predict < 1 || n_predict > SPEC_MAX_STAGES)
    return fail(SPEC_EINVAL, "n_predict = %d outside [1, %d]", n_predict, SPEC_MAX_STAGES);
  if ((int64_t)B * n_predict > kMaxTreeItems)
    return fail(SPEC_ESHAPE, "B * n_predict = %lld exceeds %d", (long long)B * n_predict, kMaxTreeItems);
  HIP_TRY(launch_tree_meta(cand_tokens, batch, B, n_predict, node_tok, node_parent, node_depth, n_nodes, cand_node, mask,
                           static_cast<hipStream_t>(hip_stream)));
  return SPEC_OK;
}

extern "C" spec_status_t spec_advance(const void* hidden, int32_t hidden_dtype, int32_t batch, int32_t B,
                                      int32_t n_predict, int32_t emb_dim, const int32_t* best_cand,
                                      const int32_t* accept_len, const int32_t* out_tokens, void* next_state,
                                      int32_t* next_tok, void* hip_stream) {
  if (!hidden || !best_cand || !accept_len || !out_tokens || !next_state || !next_tok)
    return fail(SPEC_EINVAL, "a required pointer is NULL");
  if (hidden_dtype != SPEC_F32 && hidden_dtype != SPEC_BF16)
    return fail(SPEC_EDTYPE, "hidden_dtype = %d is neither SPEC_F32 nor SPEC_BF16", hidden_dtype);
  if (batch < 1 || B < 1 || emb_dim < 1) return fail(SPEC_EINVAL, "batch, B and emb_dim must be >= 1");
  if (n_predict < 1 || n_predict > SPEC_MAX_STAGES)
    return fail(SPEC_EINVAL, "n_predict = %d outside [1, %d]", n_predict, SPEC_MAX_STAGES);
  const int64_t row_bytes = (int64_t)emb_dim * (hidden_dtype == SPEC_BF16 ? 2 : 4);
  HIP_TRY(launch_advance(hidden, row_bytes, batch, B, n_predict, best_cand, accept_len, out_tokens, next_state, next_tok,
                         static_cast<hipStream_t>(hip_stream)));
  return SPEC_OK;
}

extern "C" const char* spec_last_error(void) { return g_err; }

extern "C" spec_status_t spec_version(int32_t* major, int32_t* minor) {
  if (!major || !minor) return fail(SPEC_EINVAL, "major or minor is NULL");
  *major = 0;
  *minor = 1;
  return SPEC_OK;
}
