// C ABI of the dMoE library (declared in include/dmoe.h): validation, buffer carving, and the order in which
// the kernels of one layer pass are enqueued.  Nothing here synchronises or allocates device memory.
#include "common.h"
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

namespace dmoe {

static thread_local char g_err[512] = "";
static thread_local hipEvent_t* g_events = nullptr;
static thread_local int g_pending = DMOE_OK;   // an error found by a launcher, reported by the next launch_status()
static std::atomic<int> g_force_tile{0};
static thread_local long long* g_trace = nullptr;    // dmoe_debug_trace: buffer, capacity in items, stage to trace
static thread_local int g_trace_cap = 0, g_trace_stage = -1;

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

void fail_pending(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  g_pending = code;
}

static size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }
static bool aligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 255) == 0; }

struct Dims {
  int T, d, h, E, k, hb, db, F;
  int p_max, r_max, nnz_max, g_max, nchunks, npart;
};

static int check_config(const dmoe_config* c, Dims* out) {
  if (!c) return fail(DMOE_EINVAL, "config is NULL");
  if (c->block != kBlock) return fail(DMOE_EINVAL, "block must be 128 (got %d)", c->block);
  if (c->num_tokens < 1) return fail(DMOE_EINVAL, "num_tokens must be >= 1 (got %d)", c->num_tokens);
  if (c->d_model < kBlock || c->d_model % kBlock) return fail(DMOE_EINVAL, "d_model must be a positive multiple of 128 (got %d)", c->d_model);
  if (c->ffn_hidden < kBlock || c->ffn_hidden % kBlock) return fail(DMOE_EINVAL, "ffn_hidden must be a positive multiple of 128 (got %d)", c->ffn_hidden);
  if (c->num_experts < 1 || c->num_experts > kMaxExperts) return fail(DMOE_EINVAL, "num_experts must be in [1, %d] (got %d)", kMaxExperts, c->num_experts);
  if (c->top_k < 1 || c->top_k > kMaxTopK || c->top_k > c->num_experts) return fail(DMOE_EINVAL, "top_k must be in [1, min(num_experts, %d)] (got %d)", kMaxTopK, c->top_k);
  if (c->activation != 0 && c->activation != 1) return fail(DMOE_EINVAL, "activation must be 0 (exact GELU) or 1 (tanh form)");
  if (c->normalize_topk != 0 && c->normalize_topk != 1) return fail(DMOE_EINVAL, "normalize_topk must be 0 or 1");
  if (c->expert_capacity < 0) return fail(DMOE_EINVAL, "expert_capacity must be >= 0 (got %d)", c->expert_capacity);
  if (c->pad_to_capacity != 0 && c->pad_to_capacity != 1) return fail(DMOE_EINVAL, "pad_to_capacity must be 0 or 1");
  if (c->pad_to_capacity && c->expert_capacity == 0) return fail(DMOE_EINVAL, "pad_to_capacity needs expert_capacity > 0");
  const long long F = (long long)c->num_tokens * c->top_k;
  if (F >= (1ll << 24)) return fail(DMOE_EINVAL, "num_tokens*top_k must be below 2^24 (got %lld)", F);
  const long long wcols = (long long)c->num_experts * c->ffn_hidden;
  if (wcols * c->d_model >= (1ll << 40)) return fail(DMOE_EINVAL, "expert weights too large");
  Dims m;
  m.T = c->num_tokens; m.d = c->d_model; m.h = c->ffn_hidden; m.E = c->num_experts; m.k = c->top_k;
  m.hb = m.h / kBlock; m.db = m.d / kBlock; m.F = (int)F;
  // sum_e ceil(n_e/128)*128 <= F + 127*min(E, F), and it is a multiple of 128
  long long nonempty = m.E < F ? m.E : F;
  long long pm = ((F + 127 * nonempty) / kBlock) * kBlock;
  if (c->expert_capacity > 0) {
    // token dropping: no expert owns more than its capacity, rounded up to whole blocks
    const long long rows_cap = ((long long)c->expert_capacity + kBlock - 1) / kBlock * kBlock;
    if (c->pad_to_capacity) { pm = m.E * rows_cap;  nonempty = m.E; }
    else if (m.E * rows_cap < pm) pm = m.E * rows_cap;
    if (pm >= (1ll << 30)) return fail(DMOE_EINVAL, "num_experts*expert_capacity too large");
  }
  if (pm / kBlock * m.hb >= (1ll << 27)) return fail(DMOE_EINVAL, "too many nonzero blocks");
  m.p_max = (int)pm; m.r_max = m.p_max / kBlock; m.nnz_max = m.r_max * m.hb;
  m.g_max = (int)((m.r_max + nonempty + 1) / 2);   // sum_e ceil(rows_e / 2)
  if ((long long)m.E * m.h * kBlock >= (1ll << 31)) return fail(DMOE_EINVAL, "num_experts*ffn_hidden too large");   // byte offsets inside a 128-row slab are 32-bit
  m.nchunks = (m.F + 255) / 256;
  m.npart = router_bwd_num_partials(*c);
  if (out) *out = m;
  return DMOE_OK;
}

struct TopoLayout {
  size_t off[18];
  size_t total;
};
static TopoLayout topo_layout(const Dims& m) {
  const size_t n[18] = {
      (size_t)m.F * 4,             // expert_idx
      (size_t)m.F * 4,             // weights
      (size_t)m.T * m.E * 4,       // logits
      (size_t)m.E * 4,             // tokens_per_expert
      (size_t)(m.E + 1) * 4,       // padded_offsets
      (size_t)m.F * 4,             // row_of
      (size_t)m.p_max * 4,         // token_of
      (size_t)(m.r_max + 1) * 4,   // row_offsets
      (size_t)m.nnz_max * 4,       // column_indices
      (size_t)m.nnz_max * 4,       // row_indices
      (size_t)(m.E * m.hb + 1) * 4,// column_offsets_t
      (size_t)m.nnz_max * 4,       // row_indices_t
      (size_t)m.nnz_max * 4,       // block_offsets_t
      16,                          // counts
      (size_t)m.E * 4,             // expert_order
      (size_t)(m.E + 1) * 4,       // group_offsets
      (size_t)(m.g_max + 1) * 4,   // row_group
      16,                          // sched
  };
  TopoLayout l;
  size_t at = 0;
  for (int i = 0; i < 18; ++i) { l.off[i] = at; at += align_up(n[i]); }
  l.total = at;
  return l;
}

struct SavedLayout { size_t xp, hval, aval, yp, total; };
static SavedLayout saved_layout(const Dims& m) {
  SavedLayout l;
  const size_t pd = align_up((size_t)m.p_max * m.d * 2), bl = align_up((size_t)m.nnz_max * kBlock * kBlock * 2);
  l.xp = 0; l.hval = pd; l.aval = pd + bl; l.yp = pd + 2 * bl; l.total = 2 * pd + 2 * bl;
  return l;
}
struct ScratchLayout { size_t chunk_counts, dyp, dh, dxp, dweights, dlogits, partials, total; };
static ScratchLayout scratch_layout(const Dims& m) {
  ScratchLayout l;
  const size_t pd = align_up((size_t)m.p_max * m.d * 2), bl = align_up((size_t)m.nnz_max * kBlock * kBlock * 2);
  size_t at = 0;
  l.chunk_counts = at; at += align_up((size_t)m.nchunks * m.E * 4);
  l.dyp = at; at += pd;
  l.dh = at; at += bl;
  l.dxp = at; at += pd;
  l.dweights = at; at += align_up((size_t)m.F * 4);
  l.dlogits = at; at += align_up((size_t)m.T * m.E * 4);
  l.partials = at; at += align_up((size_t)m.npart * m.d * m.E * 4);
  l.total = at;
  return l;
}

int check_ptr(const void* p, const char* name) {
  if (!p) return fail(DMOE_EINVAL, "%s is NULL", name);
  if (!aligned(p)) return fail(DMOE_EINVAL, "%s is not 256-byte aligned", name);
  return DMOE_OK;
}
static int check_topo(const dmoe_topology_t* t) {
  if (!t) return fail(DMOE_EINVAL, "topology is NULL");
  const void* ps[18] = {t->expert_idx, t->weights, t->logits, t->tokens_per_expert, t->padded_offsets, t->row_of,
                        t->token_of, t->row_offsets, t->column_indices, t->row_indices, t->column_offsets_t,
                        t->row_indices_t, t->block_offsets_t, t->counts, t->expert_order, t->group_offsets,
                        t->row_group, t->sched};
  for (int i = 0; i < 18; ++i)
    if (!ps[i]) return fail(DMOE_EINVAL, "topology array %d is NULL (call dmoe_topology_bind first)", i);
  return DMOE_OK;
}
int launch_status() {
  const hipError_t e = hipGetLastError();
  if (g_pending != DMOE_OK) {
    const int rc = g_pending;
    g_pending = DMOE_OK;
    return rc;
  }
  if (e != hipSuccess) return fail(DMOE_ELAUNCH, "HIP error while enqueueing: %s", hipGetErrorString(e));
  return DMOE_OK;
}

}  // namespace dmoe

using namespace dmoe;

extern "C" {

int dmoe_sizes(const dmoe_config* cfg, size_t* topology_bytes, size_t* saved_bytes, size_t* scratch_bytes,
               int32_t* P_max, int32_t* nnz_max) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (topology_bytes) *topology_bytes = topo_layout(m).total;
  if (saved_bytes) *saved_bytes = saved_layout(m).total;
  if (scratch_bytes) *scratch_bytes = scratch_layout(m).total;
  if (P_max) *P_max = m.p_max;
  if (nnz_max) *nnz_max = m.nnz_max;
  return DMOE_OK;
}

int dmoe_topology_bind(const dmoe_config* cfg, void* topology_mem, size_t bytes, dmoe_topology_t* out) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (int rc = check_ptr(topology_mem, "topology_mem")) return rc;
  if (!out) return fail(DMOE_EINVAL, "out is NULL");
  const TopoLayout l = topo_layout(m);
  if (bytes < l.total) return fail(DMOE_ENOMEM, "topology buffer has %zu bytes, needs %zu", bytes, l.total);
  char* b = static_cast<char*>(topology_mem);
  out->expert_idx = reinterpret_cast<int32_t*>(b + l.off[0]);
  out->weights = reinterpret_cast<float*>(b + l.off[1]);
  out->logits = reinterpret_cast<float*>(b + l.off[2]);
  out->tokens_per_expert = reinterpret_cast<int32_t*>(b + l.off[3]);
  out->padded_offsets = reinterpret_cast<int32_t*>(b + l.off[4]);
  out->row_of = reinterpret_cast<int32_t*>(b + l.off[5]);
  out->token_of = reinterpret_cast<int32_t*>(b + l.off[6]);
  out->row_offsets = reinterpret_cast<int32_t*>(b + l.off[7]);
  out->column_indices = reinterpret_cast<int32_t*>(b + l.off[8]);
  out->row_indices = reinterpret_cast<int32_t*>(b + l.off[9]);
  out->column_offsets_t = reinterpret_cast<int32_t*>(b + l.off[10]);
  out->row_indices_t = reinterpret_cast<int32_t*>(b + l.off[11]);
  out->block_offsets_t = reinterpret_cast<int32_t*>(b + l.off[12]);
  out->counts = reinterpret_cast<int32_t*>(b + l.off[13]);
  out->expert_order = reinterpret_cast<int32_t*>(b + l.off[14]);
  out->group_offsets = reinterpret_cast<int32_t*>(b + l.off[15]);
  out->row_group = reinterpret_cast<int32_t*>(b + l.off[16]);
  out->sched = reinterpret_cast<int32_t*>(b + l.off[17]);
  return DMOE_OK;
}

int dmoe_topology(const dmoe_config* cfg, const void* x, const void* w_router, const float* router_bias,
                  dmoe_topology_t* topo, void* scratch, size_t scratch_bytes, void* stream) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (int rc = check_ptr(x, "x")) return rc;
  if (int rc = check_ptr(w_router, "w_router")) return rc;
  if (int rc = check_topo(topo)) return rc;
  if (int rc = check_ptr(scratch, "scratch")) return rc;
  const ScratchLayout sl = scratch_layout(m);
  if (scratch_bytes < sl.total) return fail(DMOE_ENOMEM, "scratch has %zu bytes, needs %zu", scratch_bytes, sl.total);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const StageEvents ev{g_events, s};
  (void)hipGetLastError();
  ev.begin(DMOE_STAGE_ROUTER);
  launch_router(*cfg, static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w_router), router_bias, *topo, s);
  ev.end(DMOE_STAGE_ROUTER);
  ev.begin(DMOE_STAGE_SORT);
  launch_sort(*cfg, *topo, reinterpret_cast<int32_t*>(static_cast<char*>(scratch) + sl.chunk_counts), m.p_max, s);
  ev.end(DMOE_STAGE_SORT);
  ev.begin(DMOE_STAGE_TOPOLOGY);
  launch_make_topology(*cfg, *topo, m.p_max, m.nnz_max, s);
  ev.end(DMOE_STAGE_TOPOLOGY);
  return launch_status();
}

// ---- dmoe_topology for callers that cannot allocate or hand over a workspace ------------------------------------
// The only scratch dmoe_topology uses is the table of per-chunk expert counts ([ceil(T*k/256)][E] int32), which the
// first grouping kernel writes in full before anything reads it, so nothing has to be cleared between calls.  Here it
// lives in a file-scope device array; the host code below never passes the array's name to the GPU (in host code that
// name is only a handle) but the device address that hipGetSymbolAddress returns for the current device.
constexpr size_t kStaticScratchBytes = (size_t)1 << 20;
static __device__ __align__(256) unsigned char static_scratch_mem[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_static_mu;
static void* g_static_ptr[kMaxDevices] = {};         // per device: each GPU holds its own copy at its own address

static int static_scratch_for_current_device(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(DMOE_ELAUNCH, "hipGetDevice failed: %s", hipGetErrorString(e));
  if (dev < 0 || dev >= kMaxDevices) return fail(DMOE_EINVAL, "device ordinal %d is outside [0, %d)", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch_mem));
    if (e != hipSuccess || !ptr)
      return fail(DMOE_ELAUNCH, "hipGetSymbolAddress(static scratch) failed on device %d: %s", dev, hipGetErrorString(e));
    g_static_ptr[dev] = ptr;
  }
  *out = g_static_ptr[dev];
  return DMOE_OK;
}

int dmoe_topology_static(const dmoe_config* cfg, const void* x, const void* w_router, const float* router_bias,
                         dmoe_topology_t* topo, void* stream) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (int rc = check_ptr(x, "x")) return rc;
  if (int rc = check_ptr(w_router, "w_router")) return rc;
  if (int rc = check_topo(topo)) return rc;
  const size_t need = (size_t)m.nchunks * m.E * 4;
  if (need > kStaticScratchBytes)
    return fail(DMOE_ENOMEM, "dmoe_topology_static: ceil(T*k/256)*E*4 = %zu bytes of chunk counts exceed the built-in "
                "%zu-byte scratch; use dmoe_topology with a caller-provided scratch", need, kStaticScratchBytes);
  void* chunk_counts = nullptr;
  if (int rc = static_scratch_for_current_device(&chunk_counts)) return rc;
  hipStream_t s = static_cast<hipStream_t>(stream);
  (void)hipGetLastError();
  launch_router(*cfg, static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w_router), router_bias, *topo, s);
  launch_sort(*cfg, *topo, static_cast<int32_t*>(chunk_counts), m.p_max, s);
  launch_make_topology(*cfg, *topo, m.p_max, m.nnz_max, s);
  return launch_status();
}

int dmoe_forward(const dmoe_config* cfg, const void* x, const void* w1, const void* w2, const dmoe_topology_t* topo,
                 void* y, void* saved, size_t saved_bytes, void* scratch, size_t scratch_bytes, void* stream) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (int rc = check_ptr(x, "x")) return rc;
  if (int rc = check_ptr(w1, "w1")) return rc;
  if (int rc = check_ptr(w2, "w2")) return rc;
  if (int rc = check_topo(topo)) return rc;
  if (int rc = check_ptr(y, "y")) return rc;
  if (int rc = check_ptr(saved, "saved")) return rc;
  (void)scratch; (void)scratch_bytes;
  const SavedLayout sv = saved_layout(m);
  if (saved_bytes < sv.total) return fail(DMOE_ENOMEM, "saved has %zu bytes, needs %zu", saved_bytes, sv.total);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const StageEvents ev{g_events, s};
  char* sb = static_cast<char*>(saved);
  bf16_t* xp = reinterpret_cast<bf16_t*>(sb + sv.xp);
  bf16_t* hval = reinterpret_cast<bf16_t*>(sb + sv.hval);
  bf16_t* aval = reinterpret_cast<bf16_t*>(sb + sv.aval);
  bf16_t* yp = reinterpret_cast<bf16_t*>(sb + sv.yp);
  (void)hipGetLastError();

  ev.begin(DMOE_STAGE_GATHER);
  launch_padded_gather(*cfg, *topo, static_cast<const bf16_t*>(x), xp, m.p_max, s);
  ev.end(DMOE_STAGE_GATHER);

  BsArgs a{};
  a.topo = topo; a.d = m.d; a.h = m.h; a.E = m.E; a.g_max = m.g_max; a.r_max = m.r_max;
  a.groups_est = (m.F + 255) / 256; a.force_tile = g_force_tile.load(std::memory_order_relaxed);
  ev.begin(DMOE_STAGE_SDD);
  a.dense_a = xp; a.dense_b = static_cast<const bf16_t*>(w1); a.sparse_in = nullptr; a.out0 = hval; a.out1 = aval;
  a.act = cfg->activation;
  a.trace = g_trace_stage == DMOE_STAGE_SDD ? g_trace : nullptr;  a.trace_cap = g_trace_cap;
  launch_bsmm(OP_SDD, a, s);
  ev.end(DMOE_STAGE_SDD);

  ev.begin(DMOE_STAGE_DSD);
  a.dense_a = nullptr; a.dense_b = static_cast<const bf16_t*>(w2); a.sparse_in = aval; a.out0 = yp; a.out1 = nullptr;
  a.trace = g_trace_stage == DMOE_STAGE_DSD ? g_trace : nullptr;  a.trace_cap = g_trace_cap;
  launch_bsmm(OP_DSD, a, s);
  ev.end(DMOE_STAGE_DSD);

  ev.begin(DMOE_STAGE_SCATTER);
  launch_weighted_scatter(*cfg, *topo, yp, static_cast<bf16_t*>(y), s);
  ev.end(DMOE_STAGE_SCATTER);
  return launch_status();
}

// dmoe_backward (accumulate = 0: bf16 weight gradients, overwritten) and dmoe_backward_accumulate (accumulate = 1:
// fp32 weight gradients, added to) differ only in the epilogue of the two weight-gradient products and in the last
// kernel of the router's gradient.
static int backward_impl(const dmoe_config* cfg, const void* x, const void* w_router, const void* w1, const void* w2,
                         const dmoe_topology_t* topo, const void* saved, size_t saved_bytes, const void* dy, void* dx,
                         void* dw_router, void* dw1, void* dw2, void* scratch, size_t scratch_bytes, void* stream,
                         int accumulate) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (int rc = check_ptr(x, "x")) return rc;
  if (int rc = check_ptr(w_router, "w_router")) return rc;
  if (int rc = check_ptr(w1, "w1")) return rc;
  if (int rc = check_ptr(w2, "w2")) return rc;
  if (int rc = check_topo(topo)) return rc;
  if (int rc = check_ptr(saved, "saved")) return rc;
  if (int rc = check_ptr(dy, "dy")) return rc;
  if (int rc = check_ptr(dx, "dx")) return rc;
  if (int rc = check_ptr(dw_router, "dw_router")) return rc;
  if (int rc = check_ptr(dw1, "dw1")) return rc;
  if (int rc = check_ptr(dw2, "dw2")) return rc;
  if (int rc = check_ptr(scratch, "scratch")) return rc;
  const SavedLayout sv = saved_layout(m);
  const ScratchLayout sl = scratch_layout(m);
  if (saved_bytes < sv.total) return fail(DMOE_ENOMEM, "saved has %zu bytes, needs %zu", saved_bytes, sv.total);
  if (scratch_bytes < sl.total) return fail(DMOE_ENOMEM, "scratch has %zu bytes, needs %zu", scratch_bytes, sl.total);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const StageEvents ev{g_events, s};
  const char* sb = static_cast<const char*>(saved);
  const bf16_t* xp = reinterpret_cast<const bf16_t*>(sb + sv.xp);
  const bf16_t* hval = reinterpret_cast<const bf16_t*>(sb + sv.hval);
  const bf16_t* aval = reinterpret_cast<const bf16_t*>(sb + sv.aval);
  const bf16_t* yp = reinterpret_cast<const bf16_t*>(sb + sv.yp);
  char* wb = static_cast<char*>(scratch);
  bf16_t* dyp = reinterpret_cast<bf16_t*>(wb + sl.dyp);
  bf16_t* dh = reinterpret_cast<bf16_t*>(wb + sl.dh);
  bf16_t* dxp = reinterpret_cast<bf16_t*>(wb + sl.dxp);
  float* dweights = reinterpret_cast<float*>(wb + sl.dweights);
  float* dlogits = reinterpret_cast<float*>(wb + sl.dlogits);
  float* partials = reinterpret_cast<float*>(wb + sl.partials);
  (void)hipGetLastError();

  ev.begin(DMOE_STAGE_BWD_GATHER);
  launch_bwd_gather(*cfg, *topo, static_cast<const bf16_t*>(dy), yp, dyp, dweights, m.p_max, s);
  ev.end(DMOE_STAGE_BWD_GATHER);

  BsArgs a{};
  a.topo = topo; a.d = m.d; a.h = m.h; a.E = m.E; a.g_max = m.g_max; a.r_max = m.r_max;
  a.groups_est = (m.F + 255) / 256; a.force_tile = g_force_tile.load(std::memory_order_relaxed);

  ev.begin(DMOE_STAGE_SDDT);   // dA = dYp W2^T on the nonzero blocks, dH = dA * G with G = gelu'(H) kept by forward
  a.dense_a = dyp; a.dense_b = static_cast<const bf16_t*>(w2); a.sparse_in = hval; a.out0 = dh; a.out1 = nullptr;
  a.trace = g_trace_stage == DMOE_STAGE_SDDT ? g_trace : nullptr;  a.trace_cap = g_trace_cap;
  launch_bsmm(OP_SDDT, a, s);
  ev.end(DMOE_STAGE_SDDT);

  ev.begin(DMOE_STAGE_DSTD);   // dW2 = A^T dYp
  a.dense_a = dyp; a.dense_b = nullptr; a.sparse_in = aval; a.out0 = static_cast<bf16_t*>(dw2);
  a.accum = accumulate;
  a.trace = g_trace_stage == DMOE_STAGE_DSTD ? g_trace : nullptr;  a.trace_cap = g_trace_cap;
  launch_bsmm(OP_DSTD, a, s);
  a.accum = 0;
  ev.end(DMOE_STAGE_DSTD);

  ev.begin(DMOE_STAGE_DSDT);   // dXp = dH W1^T
  a.dense_a = nullptr; a.dense_b = static_cast<const bf16_t*>(w1); a.sparse_in = dh; a.out0 = dxp;
  a.trace = g_trace_stage == DMOE_STAGE_DSDT ? g_trace : nullptr;  a.trace_cap = g_trace_cap;
  launch_bsmm(OP_DSDT, a, s);
  ev.end(DMOE_STAGE_DSDT);

  ev.begin(DMOE_STAGE_DDTS);   // dW1 = Xp^T dH
  a.dense_a = xp; a.dense_b = nullptr; a.sparse_in = dh; a.out0 = static_cast<bf16_t*>(dw1);
  a.accum = accumulate;
  a.trace = g_trace_stage == DMOE_STAGE_DDTS ? g_trace : nullptr;  a.trace_cap = g_trace_cap;
  launch_bsmm(OP_DDTS, a, s);
  a.accum = 0;
  ev.end(DMOE_STAGE_DDTS);

  ev.begin(DMOE_STAGE_ROUTER_BWD);
  launch_router_bwd(*cfg, *topo, static_cast<const bf16_t*>(x), static_cast<const bf16_t*>(w_router), dweights, dxp,
                    dlogits, partials, m.npart, static_cast<bf16_t*>(dx), static_cast<float*>(dw_router), accumulate != 0, s);
  ev.end(DMOE_STAGE_ROUTER_BWD);
  return launch_status();
}

int dmoe_backward(const dmoe_config* cfg, const void* x, const void* w_router, const void* w1, const void* w2,
                  const dmoe_topology_t* topo, const void* saved, size_t saved_bytes, const void* dy, void* dx,
                  void* dw_router, void* dw1, void* dw2, void* scratch, size_t scratch_bytes, void* stream) {
  return backward_impl(cfg, x, w_router, w1, w2, topo, saved, saved_bytes, dy, dx, dw_router, dw1, dw2, scratch,
                       scratch_bytes, stream, 0);
}

int dmoe_backward_accumulate(const dmoe_config* cfg, const void* x, const void* w_router, const void* w1,
                             const void* w2, const dmoe_topology_t* topo, const void* saved, size_t saved_bytes,
                             const void* dy, void* dx, float* dw_router_acc, float* dw1_acc, float* dw2_acc,
                             void* scratch, size_t scratch_bytes, void* stream) {
  return backward_impl(cfg, x, w_router, w1, w2, topo, saved, saved_bytes, dy, dx, dw_router_acc, dw1_acc, dw2_acc,
                       scratch, scratch_bytes, stream, 1);
}

int dmoe_topology_counts_host(const dmoe_topology_t* topo, int32_t* out4, void* stream) {
  if (!topo || !topo->counts || !out4) return fail(DMOE_EINVAL, "NULL argument");
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(out4, topo->counts, 16, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  if (e != hipSuccess) return fail(DMOE_ELAUNCH, "HIP error: %s", hipGetErrorString(e));
  return DMOE_OK;
}

int dmoe_debug_scratch_offset(const dmoe_config* cfg, const char* region, size_t* offset) {
  Dims m;
  if (int rc = check_config(cfg, &m)) return rc;
  if (!region || !offset) return fail(DMOE_EINVAL, "NULL argument");
  const ScratchLayout sl = scratch_layout(m);
  const struct { const char* name; size_t off; } table[] = {
      {"chunk_counts", sl.chunk_counts}, {"dyp", sl.dyp}, {"dh", sl.dh}, {"dxp", sl.dxp},
      {"dweights", sl.dweights}, {"dlogits", sl.dlogits}, {"partials", sl.partials}};
  for (const auto& t : table)
    if (strcmp(t.name, region) == 0) { *offset = t.off; return DMOE_OK; }
  return fail(DMOE_EINVAL, "unknown scratch region '%s'", region);
}

int dmoe_debug_trace(void* buffer, size_t bytes, int stage) {
  if (buffer && (reinterpret_cast<uintptr_t>(buffer) & 255)) return fail(DMOE_EINVAL, "trace buffer is not 256-byte aligned");
  if (buffer && (stage < DMOE_STAGE_SDD || stage > DMOE_STAGE_DDTS)) return fail(DMOE_EINVAL, "stage %d is not a block-sparse product", stage);
  g_trace = static_cast<long long*>(buffer);
  g_trace_cap = buffer ? (int)(bytes / 40 > 0x7fffffff ? 0x7fffffff : bytes / 40) : 0;
  g_trace_stage = buffer ? stage : -1;
  return DMOE_OK;
}

int dmoe_set_stage_events(void* events) {
  g_events = static_cast<hipEvent_t*>(events);
  return DMOE_OK;
}

int dmoe_set_tile_mode(int mode) {
  if (mode < 0 || mode > 3) return fail(DMOE_EINVAL, "tile mode must be 0 (automatic), 1 (128x128), 2 (256x256) or 3 (256x256 on two LDS stages)");
  g_force_tile.store(mode, std::memory_order_relaxed);
  return DMOE_OK;
}

const char* dmoe_last_error(void) { return g_err; }

}  // extern "C"
