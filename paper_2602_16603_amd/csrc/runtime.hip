// Host runtime behind the C ABI: model (weights, RoPE table, paged KV pool, block allocator,
// workspace cache), execution task (operator cursor, per-task workspace, preemption gate) and
// the extern "C" entry points.
//
// FlowPrefill Section 5.1: a task runs operator by operator; between operators the runtime
// looks at a signal the scheduler may have set; if set it lets the work in flight finish,
// clears the signal, acknowledges and suspends the task with all of its state left in place.
// Section 4: the execution pool keeps the state of preempted tasks until they are resumed.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <climits>
#include <cmath>
#include <condition_variable>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/flowprefill.h"
#include "common.h"
#include "kernels.h"
#include "task_core.h"

namespace {

thread_local std::string g_last_error;

fp_status fail(fp_status code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

#define FP_HIP(call)                                                                     \
  do {                                                                                   \
    hipError_t e_ = (call);                                                              \
    if (e_ != hipSuccess)                                                                \
      return fail(e_ == hipErrorOutOfMemory ? FP_ERR_OOM : FP_ERR_DEVICE, "%s: %s", #call, \
                  hipGetErrorString(e_));                                                \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

namespace fp {
void set_last_error(const char* message) { g_last_error = message; }
}  // namespace fp

namespace {

struct Workspace {
  void* base = nullptr;        // device
  size_t bytes = 0;
  void* staging = nullptr;     // pinned host memory the task's metadata is uploaded from
  size_t staging_bytes = 0;
};

using fp::kMarkRing;

}  // namespace

struct fp_model {
  fp_shape shape;
  fp::Geometry geo;
  hipStream_t stream = nullptr;
  size_t elem = 2;
  std::vector<fp_layer_weights> layers;
  float* rope_cos = nullptr;
  float* rope_sin = nullptr;
  void* k_pool = nullptr;
  void* v_pool = nullptr;
  std::mutex mu;                       // guards free_blocks, ws_cache, the event pools, live_tasks
  std::vector<int32_t> free_blocks;    // stack of free physical block ids
  std::vector<uint8_t> block_used;
  std::vector<Workspace> ws_cache;
  std::vector<hipEvent_t> marker_events;   // idle completion markers (no timing), reused by later tasks
  std::vector<hipEvent_t> timing_events;   // idle timing events
  int live_tasks = 0;
};

struct fp_prefill : fp::OpBackend {
  fp_prefill(int32_t total_ops, uint32_t mask) : core(total_ops, FP_OPS_PER_LAYER, mask) {}

  fp_model* model = nullptr;
  int32_t n_tokens = 0, n_seqs = 0, max_blocks = 0;
  std::vector<int32_t> cu, cached, tables, owned_blocks;
  Workspace ws;
  // carved out of ws:
  float* x = nullptr;
  void *h = nullptr, *qkv = nullptr, *o = nullptr, *gu = nullptr, *act = nullptr;
  // mixture-of-experts scratch (device; null for dense models)
  float* moe_logits = nullptr; float* moe_wts = nullptr;
  int32_t *moe_ids = nullptr, *moe_slot = nullptr, *moe_plan = nullptr, *moe_groups = nullptr, *moe_blocks = nullptr;
  int32_t* moe_rows = nullptr;         // token of every row of the experts' row space (gather index)
  void *moe_act = nullptr, *moe_y = nullptr;
  int32_t moe_max_row_tiles = 0;
  bool swiglu_fused = false;   // op 6 writes act directly (fused GEMM epilogue, or fused split-K reduction); op 7 then has no work and gu is not allocated
  bool swiglu_epilogue = false;   // ... by the GEMM epilogue (the problem fills the chip); else by the split-K reduction
  bool norm_after_o = false;   // short requests: op 4's split-K reduction also normalises the row (op 5 has no work)
  bool norm_after_down = false;   // ... op 8's does (op 0 of the next layer has no work)
  void* splitk = nullptr;              // split-K partial sums (0 bytes when no GEMM of this task splits)
  size_t splitk_bytes = 0;
  fp::BatchMeta meta{};
  // cursor, launch-ahead bound and preemption gate
  fp::TaskCore core;
  hipEvent_t ring[kMarkRing] = {};      // the task's own completion markers (from the model's pool)
  hipEvent_t slot_ev[kMarkRing] = {};   // event standing for marker slot i (ring[i], or a timing event)
  // per-op timing
  bool timing = false;
  std::vector<hipEvent_t> tev;          // timing events of the most recent advance call, in order
  std::vector<int32_t> tmark;           // tmark[i] = index in tev of the boundary before operator i of that call
  int32_t timed_ops = 0;

  // ---- fp::OpBackend: what the state machine asks of the device ----
  void begin_call() override;
  int launch(int32_t index, bool* launched) override;
  int mark(int slot) override;
  int wait_mark(int slot) override;
  int drain() override;
  bool wants_marks() const override { return timing; }
  void op_issued(int32_t issued, bool launched) override;
  hipEvent_t timing_event();
};

namespace {

fp_status launch_op(fp_prefill* t, int32_t index) {
  fp_model* m = t->model;
  const fp_shape& sh = m->shape;
  const int layer = index / FP_OPS_PER_LAYER, op = index % FP_OPS_PER_LAYER;
  const fp_layer_weights& w = m->layers[layer];
  const int dt = sh.dtype;
  const int64_t T = t->n_tokens, d = sh.hidden, F = sh.ffn;
  const int64_t qd = (int64_t)sh.n_q_heads * sh.head_dim;
  hipStream_t s = m->stream;
  if (sh.n_experts > 0 && op >= 6) {
    if (T == 0) return FP_OK;
    const int E = sh.n_experts, k = sh.top_k;
    int32_t* ids = t->moe_ids + (int64_t)layer * T * k;      // kept per layer for inspection
    float* wts = t->moe_wts + (int64_t)layer * T * k;
    switch (op) {
      case 6:   // gate: router logits (fp32, accumulated into zeros), selection, row plan
        fp::launch_fill_zero(t->moe_logits, T * E, s);
        fp::launch_gemm(dt, t->h, w.w_router, t->moe_logits, T, E, d, 1, t->splitk, t->splitk_bytes, s);
        fp::launch_moe_route(t->moe_logits, ids, wts, t->moe_slot, t->moe_plan, t->moe_blocks, t->moe_groups, T, E, k, s);
        break;
      case 7:   // experts, first half: gather per expert, gate/up projection + SiLU*up
        fp::launch_moe_index(ids, t->moe_plan, t->moe_blocks, t->moe_slot, t->moe_rows, T, k, E, s);
        fp::launch_gemm_grouped(t->h, w.w_gate_up, t->moe_act, F, d, 1, t->moe_groups, t->moe_max_row_tiles,
                                t->moe_rows, T, s);
        break;
      case 8:   // experts, second half: down projection, weighted sum into the residual stream
        fp::launch_gemm_grouped(t->moe_act, w.w_down, t->moe_y, d, F, 0, t->moe_groups, t->moe_max_row_tiles,
                                nullptr, 0, s);
        fp::launch_moe_combine(t->x, t->moe_y, t->moe_slot, wts, T, k, (int)d, s);
        break;
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
      return fail(FP_ERR_DEVICE, "launch of layer %d op %d failed: %s", layer, op, hipGetErrorString(e));
    return FP_OK;
  }
  switch (op) {
    case 0:
      if (!(layer > 0 && t->norm_after_down)) fp::launch_rmsnorm(dt, t->x, w.attn_norm, t->h, T, d, sh.rms_eps, s);
      break;
    case 1: fp::launch_gemm(dt, t->h, w.w_qkv, t->qkv, T, m->geo.qkv_width(), d, 0, t->splitk, t->splitk_bytes, s); break;
    case 2:
      fp::launch_rope_kvwrite(dt, t->qkv, m->rope_cos, m->rope_sin, m->geo, t->meta, layer,
                              m->k_pool, m->v_pool, s);
      break;
    case 3:
      fp::launch_attention(dt, t->qkv, m->k_pool, m->v_pool, t->o, m->geo, t->meta, layer, s);
      break;
    case 4: {
      fp::GemmTail tail;
      if (t->norm_after_o) tail = fp::GemmTail{fp::kTailRmsNorm, w.mlp_norm, t->h, sh.rms_eps};
      fp::launch_gemm(dt, t->o, w.w_o, t->x, T, d, qd, 1, t->splitk, t->splitk_bytes, s, &tail);
      break;
    }
    case 5:
      if (!t->norm_after_o) fp::launch_rmsnorm(dt, t->x, w.mlp_norm, t->h, T, d, sh.rms_eps, s);
      break;
    case 6:
      if (t->swiglu_epilogue) {
        fp::launch_gemm_swiglu(t->h, w.w_gate_up, t->act, T, F, d, s);
      } else {
        fp::GemmTail tail;
        if (t->swiglu_fused) tail = fp::GemmTail{fp::kTailSwiGLU, nullptr, t->act, 0.f};
        fp::launch_gemm(dt, t->h, w.w_gate_up, t->gu, T, 2 * F, d, 0, t->splitk, t->splitk_bytes, s, &tail);
      }
      break;
    case 7:
      if (!t->swiglu_fused) fp::launch_silu_mul(dt, t->gu, t->act, T, F, s);
      break;
    case 8: {
      fp::GemmTail tail;
      if (t->norm_after_down && layer + 1 < sh.n_layers)
        tail = fp::GemmTail{fp::kTailRmsNorm, m->layers[layer + 1].attn_norm, t->h, sh.rms_eps};
      fp::launch_gemm(dt, t->act, w.w_down, t->x, T, d, F, 1, t->splitk, t->splitk_bytes, s, &tail);
      break;
    }
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess)
    return fail(FP_ERR_DEVICE, "launch of layer %d op %d failed: %s", layer, op,
                hipGetErrorString(e));
  return FP_OK;
}

// Device workspace + pinned staging for one task.  Workspaces are cached in the model: a request
// takes the smallest cached one that fits; on a miss every cached one (all too small) is freed
// before the new allocation, so the cache never holds more than the tasks in flight need.
fp_status acquire_workspace(fp_model* m, size_t bytes, size_t staging_bytes, Workspace* out) {
  std::vector<Workspace> drop;
  Workspace got;
  {
    std::lock_guard<std::mutex> lk(m->mu);
    int best = -1;
    for (int i = 0; i < (int)m->ws_cache.size(); ++i)
      if (m->ws_cache[i].bytes >= bytes && (best < 0 || m->ws_cache[i].bytes < m->ws_cache[best].bytes))
        best = i;
    if (best >= 0) {
      got = m->ws_cache[best];
      m->ws_cache.erase(m->ws_cache.begin() + best);
    } else {
      drop.swap(m->ws_cache);
    }
  }
  for (auto& w : drop) {          // idle since their task ended (which drained the stream)
    (void)hipFree(w.base);
    (void)hipHostFree(w.staging);
  }
  if (!got.base) {
    FP_HIP(hipMalloc(&got.base, bytes));
    got.bytes = bytes;
  }
  if (got.staging_bytes < staging_bytes) {
    (void)hipHostFree(got.staging);
    got.staging = nullptr;
    got.staging_bytes = 0;
    const size_t want = std::max<size_t>(staging_bytes, 64 << 10);
    hipError_t e = hipHostMalloc(&got.staging, want, hipHostMallocDefault);
    if (e != hipSuccess) {
      (void)hipFree(got.base);
      return fail(FP_ERR_OOM, "pinned staging buffer: %s", hipGetErrorString(e));
    }
    got.staging_bytes = want;
  }
  *out = got;
  return FP_OK;
}

void release_workspace(fp_model* m, Workspace ws) {
  if (!ws.base) return;
  std::lock_guard<std::mutex> lk(m->mu);
  m->ws_cache.push_back(ws);
}

// Events are pooled in the model: creating and destroying eight of them per task showed up in the
// time of short requests.
fp_status acquire_events(fp_model* m, bool with_timing, int n, hipEvent_t* out) {
  std::vector<hipEvent_t>& pool = with_timing ? m->timing_events : m->marker_events;
  int got = 0;
  {
    std::lock_guard<std::mutex> lk(m->mu);
    while (got < n && !pool.empty()) { out[got++] = pool.back(); pool.pop_back(); }
  }
  for (; got < n; ++got) {
    hipError_t e = with_timing ? hipEventCreate(&out[got]) : hipEventCreateWithFlags(&out[got], hipEventDisableTiming);
    if (e != hipSuccess) {
      for (int i = 0; i < got; ++i) (void)hipEventDestroy(out[i]);
      return fail(FP_ERR_DEVICE, "event creation: %s", hipGetErrorString(e));
    }
  }
  return FP_OK;
}

void release_events(fp_model* m, bool with_timing, int n, hipEvent_t* ev) {
  std::lock_guard<std::mutex> lk(m->mu);
  std::vector<hipEvent_t>& pool = with_timing ? m->timing_events : m->marker_events;
  for (int i = 0; i < n; ++i)
    if (ev[i]) { pool.push_back(ev[i]); ev[i] = nullptr; }
}

}  // namespace

// ---- the task as the state machine's device backend ----
hipEvent_t fp_prefill::timing_event() {
  hipEvent_t ev = nullptr;
  if (acquire_events(model, true, 1, &ev) != FP_OK) return nullptr;
  tev.push_back(ev);
  (void)hipEventRecord(ev, model->stream);
  return ev;
}

void fp_prefill::begin_call() {
  timed_ops = 0;
  if (!timing) return;
  release_events(model, true, (int)tev.size(), tev.data());
  tev.clear();
  tmark.assign(1, 0);
  (void)timing_event();
}

int fp_prefill::launch(int32_t index, bool* launched) {
  const int op = index % FP_OPS_PER_LAYER;
  *launched = !((swiglu_fused && op == 7) || (norm_after_o && op == 5) ||
                (norm_after_down && op == 0 && index >= FP_OPS_PER_LAYER));
  return launch_op(this, index) == FP_OK ? 0 : -1;
}

// One event per operator serves both the launch-ahead bound and the timing read-out (an event
// record costs the device a few microseconds between two kernels).
int fp_prefill::mark(int slot) {
  hipEvent_t ev = ring[slot];
  if (timing) {
    ev = timing_event();
    if (!ev) return -1;
  } else {
    hipError_t e = hipEventRecord(ev, model->stream);
    if (e != hipSuccess) { fail(FP_ERR_DEVICE, "event record: %s", hipGetErrorString(e)); return -1; }
  }
  slot_ev[slot] = ev;
  return 0;
}

int fp_prefill::wait_mark(int slot) {
  hipError_t e = hipEventSynchronize(slot_ev[slot]);
  if (e != hipSuccess) { fail(FP_ERR_DEVICE, "event wait: %s", hipGetErrorString(e)); return -1; }
  return 0;
}

int fp_prefill::drain() {
  hipError_t e = hipStreamSynchronize(model->stream);
  if (e != hipSuccess) { fail(FP_ERR_DEVICE, "stream sync: %s", hipGetErrorString(e)); return -1; }
  return 0;
}

void fp_prefill::op_issued(int32_t issued, bool /*launched*/) {
  if (!timing) return;
  tmark.push_back((int32_t)tev.size() - 1);
  timed_ops = issued + 1;
}

extern "C" {

const char* fp_last_error(void) { return g_last_error.c_str(); }
const char* fp_version(void) { return "flowprefill-gfx950 0.1"; }

fp_status fp_model_create(const fp_shape* shape, const fp_layer_weights* layers, void* hip_stream,
                          fp_model** out) {
  if (!shape || !layers || !out) return fail(FP_ERR_INVALID, "null argument");
  const fp_shape& s = *shape;
  if (s.n_layers <= 0 || s.hidden <= 0 || s.n_q_heads <= 0 || s.n_kv_heads <= 0 ||
      s.head_dim <= 0 || s.ffn <= 0 || s.kv_num_blocks <= 0 || s.max_position <= 0)
    return fail(FP_ERR_INVALID, "non-positive shape field");
  if (s.dtype != FP_DTYPE_F32 && s.dtype != FP_DTYPE_BF16)
    return fail(FP_ERR_INVALID, "dtype must be 0 (fp32) or 1 (bf16)");
  if (s.kv_block_tokens != fp::kKvBlock) return fail(FP_ERR_INVALID, "kv_block_tokens must be 16");
  if (s.n_q_heads % s.n_kv_heads) return fail(FP_ERR_INVALID, "n_q_heads not a multiple of n_kv_heads");
  if (s.hidden % 8 || s.ffn % 8 || s.head_dim % 16)
    return fail(FP_ERR_INVALID, "hidden and ffn must be multiples of 8, head_dim of 16");
  if (s.dtype == FP_DTYPE_BF16 && s.head_dim != 64 && s.head_dim != 128)
    return fail(FP_ERR_INVALID, "bf16 path supports head_dim 64 or 128");
  if (s.dtype == FP_DTYPE_F32 && s.head_dim != 16 && s.head_dim != 32 && s.head_dim != 64 &&
      s.head_dim != 128)
    return fail(FP_ERR_INVALID, "fp32 path supports head_dim 16, 32, 64 or 128");
  if (s.kv_num_blocks > INT32_MAX) return fail(FP_ERR_INVALID, "kv_num_blocks too large");
  if (s.n_experts < 0 || s.top_k < 0 || (s.n_experts == 0) != (s.top_k == 0))
    return fail(FP_ERR_INVALID, "n_experts and top_k must both be zero (dense) or both positive");
  if (s.n_experts > 0) {
    if (s.dtype != FP_DTYPE_BF16) return fail(FP_ERR_INVALID, "mixture-of-experts models are bf16 only");
    if (s.n_experts > 256 || s.n_experts % 8 || s.top_k > 8 || s.top_k > s.n_experts)
      return fail(FP_ERR_INVALID, "n_experts must be a multiple of 8 up to 256, top_k at most 8 and n_experts");
    if (s.hidden % 64 || s.ffn % 64)
      return fail(FP_ERR_INVALID, "mixture-of-experts models need hidden and ffn multiples of 64");
  }
  for (int l = 0; l < s.n_layers; ++l) {
    const void* ptrs[7] = {layers[l].attn_norm, layers[l].w_qkv, layers[l].w_o, layers[l].mlp_norm,
                           layers[l].w_gate_up, layers[l].w_down, layers[l].w_router};
    for (int i = 0; i < (s.n_experts > 0 ? 7 : 6); ++i)
      if (!ptrs[i] || (reinterpret_cast<uintptr_t>(ptrs[i]) & 15))
        return fail(FP_ERR_INVALID, "layer %d: null or misaligned weight pointer", l);
  }
  fp_model* m = new (std::nothrow) fp_model();
  if (!m) return fail(FP_ERR_OOM, "host allocation failed");
  m->shape = s;
  m->geo = fp::Geometry{s.hidden, s.n_q_heads, s.n_kv_heads, s.head_dim, s.ffn, s.kv_num_blocks};
  m->stream = reinterpret_cast<hipStream_t>(hip_stream);
  m->elem = s.dtype == FP_DTYPE_BF16 ? 2 : 4;
  m->layers.assign(layers, layers + s.n_layers);

  // RoPE table: angle = p * theta^(-2j/D), evaluated in fp64 and rounded once to fp32.
  const int half = s.head_dim / 2;
  std::vector<float> hc((size_t)s.max_position * half), hs((size_t)s.max_position * half);
  std::vector<double> inv_freq(half);
  for (int j = 0; j < half; ++j)
    inv_freq[j] = std::pow((double)s.rope_theta, -2.0 * (double)j / (double)s.head_dim);
  for (int64_t p = 0; p < s.max_position; ++p)
    for (int j = 0; j < half; ++j) {
      const double ang = (double)p * inv_freq[j];
      hc[(size_t)p * half + j] = (float)std::cos(ang);
      hs[(size_t)p * half + j] = (float)std::sin(ang);
    }
  const size_t tbytes = hc.size() * sizeof(float);
  const size_t pool_bytes = (size_t)s.n_layers * (size_t)s.kv_num_blocks * s.n_kv_heads *
                            fp::kKvBlock * s.head_dim * m->elem;
  auto cleanup = [&]() {
    (void)hipFree(m->rope_cos); (void)hipFree(m->rope_sin);
    (void)hipFree(m->k_pool); (void)hipFree(m->v_pool);
    delete m;
  };
  hipError_t e;
  if ((e = hipMalloc((void**)&m->rope_cos, tbytes)) != hipSuccess ||
      (e = hipMalloc((void**)&m->rope_sin, tbytes)) != hipSuccess ||
      (e = hipMalloc(&m->k_pool, pool_bytes)) != hipSuccess ||
      (e = hipMalloc(&m->v_pool, pool_bytes)) != hipSuccess) {
    cleanup();
    return fail(e == hipErrorOutOfMemory ? FP_ERR_OOM : FP_ERR_DEVICE, "model allocation: %s",
                hipGetErrorString(e));
  }
  // The pools start at zero so that never-written slots of a partially filled block hold finite
  // values (the attention kernel multiplies them by an exact zero weight).
  if ((e = hipMemcpy(m->rope_cos, hc.data(), tbytes, hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipMemcpy(m->rope_sin, hs.data(), tbytes, hipMemcpyHostToDevice)) != hipSuccess ||
      (e = hipMemset(m->k_pool, 0, pool_bytes)) != hipSuccess ||
      (e = hipMemset(m->v_pool, 0, pool_bytes)) != hipSuccess ||
      (e = hipDeviceSynchronize()) != hipSuccess) {
    cleanup();
    return fail(FP_ERR_DEVICE, "model initialisation: %s", hipGetErrorString(e));
  }
  m->free_blocks.resize((size_t)s.kv_num_blocks);
  for (int64_t i = 0; i < s.kv_num_blocks; ++i)
    m->free_blocks[(size_t)i] = (int32_t)(s.kv_num_blocks - 1 - i);   // pop gives 0,1,2,...
  m->block_used.assign((size_t)s.kv_num_blocks, 0);
  *out = m;
  return FP_OK;
}

void fp_model_destroy(fp_model* m) {
  if (!m) return;
  {
    std::lock_guard<std::mutex> lk(m->mu);
    if (m->live_tasks > 0) {
      // Freeing the pools under tasks that still point into them would be a use after free on the
      // device: refuse, leave the model intact, and say so.
      char buf[128];
      snprintf(buf, sizeof(buf), "fp_model_destroy: %d task(s) not ended; model left alive", m->live_tasks);
      g_last_error = buf;
      return;
    }
  }
  (void)hipStreamSynchronize(m->stream);
  for (auto& ws : m->ws_cache) { (void)hipFree(ws.base); (void)hipHostFree(ws.staging); }
  for (auto& ev : m->marker_events) (void)hipEventDestroy(ev);
  for (auto& ev : m->timing_events) (void)hipEventDestroy(ev);
  (void)hipFree(m->rope_cos);
  (void)hipFree(m->rope_sin);
  (void)hipFree(m->k_pool);
  (void)hipFree(m->v_pool);
  delete m;
}

fp_status fp_kv_alloc(fp_model* m, int32_t n, int32_t* ids_out) {
  if (!m || n < 0 || (n > 0 && !ids_out)) return fail(FP_ERR_INVALID, "bad argument");
  std::lock_guard<std::mutex> lk(m->mu);
  if ((size_t)n > m->free_blocks.size())
    return fail(FP_ERR_OOM, "KV pool exhausted: %d blocks wanted, %zu free", n, m->free_blocks.size());
  for (int i = 0; i < n; ++i) {
    ids_out[i] = m->free_blocks.back();
    m->free_blocks.pop_back();
    m->block_used[(size_t)ids_out[i]] = 1;
  }
  return FP_OK;
}

fp_status fp_kv_free(fp_model* m, int32_t n, const int32_t* ids) {
  if (!m || n < 0 || (n > 0 && !ids)) return fail(FP_ERR_INVALID, "bad argument");
  std::lock_guard<std::mutex> lk(m->mu);
  for (int i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= m->shape.kv_num_blocks || !m->block_used[(size_t)ids[i]])
      return fail(FP_ERR_INVALID, "block %d is not allocated", ids[i]);
  for (int i = 0; i < n; ++i) {
    m->block_used[(size_t)ids[i]] = 0;
    m->free_blocks.push_back(ids[i]);
  }
  return FP_OK;
}

fp_status fp_model_kv_pools(const fp_model* m, const void** k_pool, const void** v_pool) {
  if (!m || !k_pool || !v_pool) return fail(FP_ERR_INVALID, "null argument");
  *k_pool = m->k_pool;
  *v_pool = m->v_pool;
  return FP_OK;
}

fp_status fp_prefill_begin(fp_model* m, const void* hidden_in, const int32_t* cu_seqlens,
                           int32_t n_seqs, const int32_t* cached_lens, const int32_t* block_tables,
                           int32_t max_blocks, uint32_t boundary_mask, fp_prefill** out) {
  if (!m || !cu_seqlens || !out || n_seqs < 0) return fail(FP_ERR_INVALID, "null or negative argument");
  if (cu_seqlens[0] != 0) return fail(FP_ERR_INVALID, "cu_seqlens[0] must be 0");
  for (int s = 0; s < n_seqs; ++s)
    if (cu_seqlens[s + 1] < cu_seqlens[s]) return fail(FP_ERR_INVALID, "cu_seqlens decreases at %d", s);
  const int32_t T = cu_seqlens[n_seqs];
  if (T > 0 && (!hidden_in || (reinterpret_cast<uintptr_t>(hidden_in) & 15)))
    return fail(FP_ERR_INVALID, "hidden_in null or not 16-byte aligned");
  if (!block_tables && cached_lens)
    for (int s = 0; s < n_seqs; ++s)
      if (cached_lens[s] != 0)
        return fail(FP_ERR_INVALID, "cached_lens needs caller-provided block_tables");
  if (block_tables && max_blocks <= 0) return fail(FP_ERR_INVALID, "max_blocks must be positive");
  const fp_shape& sh = m->shape;
  if (sh.n_experts > 0 && (int64_t)T * sh.hidden >= (int64_t)1 << 30)
    return fail(FP_ERR_INVALID, "mixture-of-experts task of %d tokens: tokens x hidden must stay below 2^30 "
                                "(the experts' GEMM gathers activation rows through 32-bit offsets)", T);

  fp_prefill* t = new (std::nothrow) fp_prefill(sh.n_layers * FP_OPS_PER_LAYER, boundary_mask & FP_BOUNDARY_EVERY_OP);
  if (!t) return fail(FP_ERR_OOM, "host allocation failed");
  t->model = m;
  t->n_tokens = T;
  t->n_seqs = n_seqs;
  t->cu.assign(cu_seqlens, cu_seqlens + n_seqs + 1);
  t->cached.assign((size_t)n_seqs, 0);
  if (cached_lens) t->cached.assign(cached_lens, cached_lens + n_seqs);

  std::vector<int32_t> need((size_t)n_seqs, 0);
  int32_t need_max = 1;
  for (int s = 0; s < n_seqs; ++s) {
    const int64_t len = (int64_t)t->cached[s] + (t->cu[s + 1] - t->cu[s]);
    if (t->cached[s] < 0 || len > sh.max_position) {
      delete t;
      return fail(FP_ERR_INVALID, "sequence %d: %lld positions exceed max_position %d", s,
                  (long long)len, sh.max_position);
    }
    need[s] = (int32_t)((len + fp::kKvBlock - 1) / fp::kKvBlock);
    need_max = std::max(need_max, need[s]);
  }
  if (block_tables) {
    if (max_blocks < need_max && T > 0) {
      delete t;
      return fail(FP_ERR_INVALID, "max_blocks %d < %d blocks needed", max_blocks, need_max);
    }
    t->max_blocks = max_blocks;
    t->tables.assign(block_tables, block_tables + (size_t)n_seqs * max_blocks);
    for (int s = 0; s < n_seqs; ++s)
      for (int b = 0; b < need[s]; ++b) {
        const int32_t id = t->tables[(size_t)s * max_blocks + b];
        if (id < 0 || id >= sh.kv_num_blocks) {
          delete t;
          return fail(FP_ERR_INVALID, "sequence %d block %d: id %d outside the pool", s, b, id);
        }
      }
  } else {
    t->max_blocks = need_max;
    t->tables.assign((size_t)n_seqs * need_max, -1);
    int64_t total = 0;
    for (int s = 0; s < n_seqs; ++s) total += need[s];
    t->owned_blocks.resize((size_t)total);
    fp_status st = fp_kv_alloc(m, (int32_t)total, t->owned_blocks.data());
    if (st != FP_OK) { delete t; return st; }
    size_t at = 0;
    for (int s = 0; s < n_seqs; ++s)
      for (int b = 0; b < need[s]; ++b) t->tables[(size_t)s * need_max + b] = t->owned_blocks[at++];
  }

  // ---- host-side work lists ----
  const int bqw = fp::attention_q_tile_rows(sh.head_dim);
  std::vector<int32_t> tok_seq((size_t)T), tok_pos((size_t)T), kv_items, attn_items;
  struct Item { int32_t seq, qt, work; };
  std::vector<Item> items;
  for (int s = 0; s < n_seqs; ++s) {
    const int32_t lo = t->cu[s], n = t->cu[s + 1] - lo, c = t->cached[s];
    for (int i = 0; i < n; ++i) { tok_seq[(size_t)lo + i] = s; tok_pos[(size_t)lo + i] = c + i; }
    if (n == 0) continue;
    for (int32_t lb = c / fp::kKvBlock; lb <= (c + n - 1) / fp::kKvBlock; ++lb) {
      kv_items.push_back(s);
      kv_items.push_back(lb);
    }
    for (int32_t qt = 0; qt * bqw < n; ++qt) {
      const int32_t kv_len = c + std::min(n, (qt + 1) * bqw);
      items.push_back(Item{s, qt, (kv_len + 63) / 64});
    }
  }
  // Longest first: workgroups are dispatched in index order, so the heaviest causal tiles
  // start first and the short ones fill the tail.
  std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) { return a.work > b.work; });
  for (const Item& it : items) { attn_items.push_back(it.seq); attn_items.push_back(it.qt); }

  // ---- workspace layout ----
  const size_t e = m->elem;
  const size_t d = sh.hidden, W = (size_t)m->geo.qkv_width(), qd = (size_t)sh.n_q_heads * sh.head_dim,
               F = sh.ffn;
  const size_t Tn = (size_t)std::max(T, 1);
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t o = off; off += align_up(bytes, 256); return o; };
  const bool moe = sh.n_experts > 0;
  const size_t E = (size_t)sh.n_experts, pairs = Tn * (size_t)sh.top_k;
  // Split-K workspace first: which operators fuse depends on whether their GEMM will be cut.
  const size_t sk_dense = std::max(fp::gemm_workspace_bytes(sh.dtype, T, 2 * (int64_t)F, (int64_t)d),
                                   fp::gemm_workspace_bytes(sh.dtype, T, (int64_t)d, (int64_t)F));
  const size_t sk_bytes = std::max(
      std::max(fp::gemm_workspace_bytes(sh.dtype, T, (int64_t)W, (int64_t)d), fp::gemm_workspace_bytes(sh.dtype, T, (int64_t)d, (int64_t)qd)),
      moe ? fp::gemm_workspace_bytes(sh.dtype, T, (int64_t)E, (int64_t)d) : sk_dense);
  t->swiglu_epilogue = !moe && fp::gemm_swiglu_fusable(sh.dtype, T, (int64_t)F, (int64_t)d);
  t->swiglu_fused = t->swiglu_epilogue ||
                    (!moe && fp::gemm_tail_fusable(sh.dtype, T, 2 * (int64_t)F, (int64_t)d, sk_bytes, fp::kTailSwiGLU));
  t->norm_after_o = fp::gemm_tail_fusable(sh.dtype, T, (int64_t)d, (int64_t)qd, sk_bytes, fp::kTailRmsNorm);
  t->norm_after_down = !moe && fp::gemm_tail_fusable(sh.dtype, T, (int64_t)d, (int64_t)F, sk_bytes, fp::kTailRmsNorm);
  const size_t o_x = carve(Tn * d * 4), o_h = carve(Tn * d * e), o_qkv = carve(Tn * W * e),
               o_o = carve(Tn * qd * e), o_gu = carve(t->swiglu_fused || moe ? 0 : Tn * 2 * F * e),
               o_act = carve(moe ? 0 : Tn * F * e);
  // Mixture-of-experts scratch: every (token, choice) pair owns one row of the gathered buffers.
  t->moe_max_row_tiles = moe ? (int32_t)(pairs / 256 + E) : 0;
  const size_t o_ml = carve(moe ? Tn * E * 4 : 0), o_mw = carve(moe ? pairs * 4 * sh.n_layers : 0),
               o_mi = carve(moe ? pairs * 4 * sh.n_layers : 0), o_ms = carve(moe ? pairs * 4 : 0),
               o_mp = carve(moe ? E * 4 : 0), o_mb = carve(moe ? (size_t)fp::moe_route_blocks(T) * E * 4 : 0), o_mg = carve(moe ? (1 + 3 * (size_t)t->moe_max_row_tiles) * 4 : 0),
               o_mh = carve(moe ? pairs * 4 : 0), o_ma = carve(moe ? pairs * F * e : 0),
               o_my = carve(moe ? pairs * d * e : 0);
  const size_t o_sk = carve(sk_bytes);
  const size_t n_int = tok_seq.size() + tok_pos.size() + t->cu.size() + t->cached.size() +
                       t->tables.size() + kv_items.size() + attn_items.size();
  const size_t o_int = carve((n_int + 16) * 4);
  fp_status st = acquire_workspace(m, off, (n_int + 16) * 4, &t->ws);
  if (st != FP_OK) {
    if (!t->owned_blocks.empty()) fp_kv_free(m, (int32_t)t->owned_blocks.size(), t->owned_blocks.data());
    delete t;
    return st;
  }
  char* base = static_cast<char*>(t->ws.base);
  t->x = reinterpret_cast<float*>(base + o_x);
  t->splitk = sk_bytes ? base + o_sk : nullptr; t->splitk_bytes = sk_bytes;
  t->h = base + o_h; t->qkv = base + o_qkv; t->o = base + o_o; t->gu = base + o_gu; t->act = base + o_act;
  if (moe) {
    t->moe_logits = reinterpret_cast<float*>(base + o_ml); t->moe_wts = reinterpret_cast<float*>(base + o_mw);
    t->moe_ids = reinterpret_cast<int32_t*>(base + o_mi); t->moe_slot = reinterpret_cast<int32_t*>(base + o_ms);
    t->moe_plan = reinterpret_cast<int32_t*>(base + o_mp); t->moe_blocks = reinterpret_cast<int32_t*>(base + o_mb); t->moe_groups = reinterpret_cast<int32_t*>(base + o_mg);
    t->moe_rows = reinterpret_cast<int32_t*>(base + o_mh); t->moe_act = base + o_ma; t->moe_y = base + o_my;
  }

  // Metadata goes through the workspace's pinned staging buffer, so the upload is asynchronous
  // and nothing here waits for the stream.
  int32_t* ints = static_cast<int32_t*>(t->ws.staging);
  size_t n_put = 0;
  auto put = [&](const std::vector<int32_t>& v) {
    const size_t at = n_put;
    if (!v.empty()) memcpy(ints + at, v.data(), v.size() * 4);
    n_put += v.size();
    return at;
  };
  const size_t a_seq = put(tok_seq), a_pos = put(tok_pos), a_cu = put(t->cu), a_cached = put(t->cached),
               a_tab = put(t->tables), a_kv = put(kv_items), a_attn = put(attn_items);
  int32_t* dints = reinterpret_cast<int32_t*>(base + o_int);
  auto bail = [&](fp_status code) {
    (void)hipStreamSynchronize(m->stream);      // nothing of this task may still be in flight
    release_workspace(m, t->ws);
    if (!t->owned_blocks.empty()) fp_kv_free(m, (int32_t)t->owned_blocks.size(), t->owned_blocks.data());
    release_events(m, false, kMarkRing, t->ring);
    delete t;
    return code;
  };
  hipError_t he;
  if (n_put &&
      (he = hipMemcpyAsync(dints, ints, n_put * 4, hipMemcpyHostToDevice, m->stream)) != hipSuccess)
    return bail(fail(FP_ERR_DEVICE, "metadata upload: %s", hipGetErrorString(he)));
  t->meta.n_tokens = T;
  t->meta.n_seqs = n_seqs;
  t->meta.max_blocks = t->max_blocks;
  t->meta.tok_seq = dints + a_seq;
  t->meta.tok_pos = dints + a_pos;
  t->meta.cu_seqlens = dints + a_cu;
  t->meta.cached_lens = dints + a_cached;
  t->meta.block_tables = dints + a_tab;
  t->meta.kv_items = dints + a_kv;
  t->meta.n_kv_items = (int32_t)(kv_items.size() / 2);
  t->meta.attn_items = dints + a_attn;
  t->meta.n_attn_items = (int32_t)(attn_items.size() / 2);

  fp::launch_to_residual(sh.dtype, hidden_in, t->x, (int64_t)T * sh.hidden, m->stream);
  if ((he = hipGetLastError()) != hipSuccess)
    return bail(fail(FP_ERR_DEVICE, "residual initialisation: %s", hipGetErrorString(he)));
  if ((st = acquire_events(m, false, kMarkRing, t->ring)) != FP_OK) return bail(st);
  {
    std::lock_guard<std::mutex> lk(m->mu);
    m->live_tasks++;
  }
  *out = t;
  return FP_OK;
}

fp_status fp_prefill_set_launch_ahead(fp_prefill* t, int32_t k) {
  if (!t) return fail(FP_ERR_INVALID, "null task");
  switch (t->core.set_launch_ahead(k)) {
    case fp::kTaskOk: return FP_OK;
    case fp::kTaskErrState: return fail(FP_ERR_STATE, "task is running");
    default: return fail(FP_ERR_INVALID, "launch_ahead must be 0..%d", kMarkRing);
  }
}

fp_status fp_prefill_set_timing(fp_prefill* t, int32_t on) {
  if (!t) return fail(FP_ERR_INVALID, "null task");
  if (!t->core.unless_running([&] { t->timing = on != 0; })) return fail(FP_ERR_STATE, "task is running");
  return FP_OK;
}

fp_status fp_prefill_advance(fp_prefill* t, int32_t max_ops, int32_t* ops_done) {
  if (!t || max_ops < 0) return fail(FP_ERR_INVALID, "bad argument");
  const int r = t->core.advance(*t, max_ops, ops_done);
  if (r == fp::kTaskErrState) {
    const fp::TaskState st = t->core.state();
    return fail(FP_ERR_STATE, "advance on a task that is %s",
                st == fp::TaskState::Parked ? "parked" : st == fp::TaskState::Done ? "done" : "running");
  }
  return static_cast<fp_status>(r);       // device errors: the backend has set the message
}

fp_status fp_preempt_signal(fp_prefill* t) {
  if (!t) return fail(FP_ERR_INVALID, "null task");
  const int r = t->core.preempt_signal();
  if (r == fp::kTaskErrState) return fail(FP_ERR_STATE, "task is already parked");
  return static_cast<fp_status>(r);
}

fp_status fp_preempt_wait(fp_prefill* t) {
  if (!t) return fail(FP_ERR_INVALID, "null task");
  const int r = t->core.preempt_wait();
  if (r == fp::kTaskErrState) return fail(FP_ERR_STATE, "no preemption pending on an idle task");
  return static_cast<fp_status>(r);
}

fp_status fp_preempt(fp_prefill* t) {
  fp_status st = fp_preempt_signal(t);
  if (st != FP_OK) return st;
  return fp_preempt_wait(t);
}

fp_status fp_resume(fp_prefill* t) {
  if (!t) return fail(FP_ERR_INVALID, "null task");
  if (t->core.resume() != fp::kTaskOk) return fail(FP_ERR_STATE, "resume of a task that is not parked");
  return FP_OK;
}

fp_status fp_prefill_cursor(const fp_prefill* t, int32_t* layer, int32_t* op) {
  if (!t || !layer || !op) return fail(FP_ERR_INVALID, "null argument");
  const int32_t c = t->core.cursor();      // atomic: may be polled while another thread advances
  *layer = c / FP_OPS_PER_LAYER;
  *op = c % FP_OPS_PER_LAYER;
  return FP_OK;
}

fp_status fp_prefill_hidden(const fp_prefill* t, const void** dev_ptr) {
  if (!t || !dev_ptr) return fail(FP_ERR_INVALID, "null argument");
  *dev_ptr = t->x;
  return FP_OK;
}

fp_status fp_prefill_block_tables(const fp_prefill* t, const int32_t** tables_host, int32_t* max_blocks) {
  if (!t || !tables_host || !max_blocks) return fail(FP_ERR_INVALID, "null argument");
  *tables_host = t->tables.data();
  *max_blocks = t->max_blocks;
  return FP_OK;
}

fp_status fp_prefill_kv(const fp_prefill* t, int32_t layer, const void** k_pool, const void** v_pool,
                        const int32_t** block_tables_host) {
  if (!t || !k_pool || !v_pool || !block_tables_host) return fail(FP_ERR_INVALID, "null argument");
  const fp_model* m = t->model;
  if (layer < 0 || layer >= m->shape.n_layers) return fail(FP_ERR_INVALID, "layer out of range");
  const size_t layer_bytes = (size_t)m->shape.kv_num_blocks * m->shape.n_kv_heads * fp::kKvBlock *
                             m->shape.head_dim * m->elem;
  *k_pool = static_cast<const char*>(m->k_pool) + (size_t)layer * layer_bytes;
  *v_pool = static_cast<const char*>(m->v_pool) + (size_t)layer * layer_bytes;
  *block_tables_host = t->tables.data();
  return FP_OK;
}

fp_status fp_prefill_kv_gather(const fp_prefill* t, int32_t layer, int32_t seq, void* k_out, void* v_out) {
  if (!t || !k_out || !v_out) return fail(FP_ERR_INVALID, "null argument");
  const fp_model* m = t->model;
  if (layer < 0 || layer >= m->shape.n_layers || seq < 0 || seq >= t->n_seqs)
    return fail(FP_ERR_INVALID, "layer or sequence out of range");
  const int len = t->cached[seq] + (t->cu[seq + 1] - t->cu[seq]);
  fp::launch_kv_gather(m->shape.dtype, m->k_pool, m->v_pool, k_out, v_out, len, m->geo, layer,
                       t->meta.block_tables + (size_t)seq * t->max_blocks, m->stream);
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipStreamSynchronize(m->stream);
  return e == hipSuccess ? FP_OK : fail(FP_ERR_DEVICE, "kv gather: %s", hipGetErrorString(e));
}

fp_status fp_prefill_op_times(fp_prefill* t, float* ms_out, int32_t n, int32_t* n_out) {
  if (!t || !ms_out || !n_out || n < 0) return fail(FP_ERR_INVALID, "bad argument");
  const int32_t cnt = std::min(n, t->timed_ops);
  for (int32_t i = 0; i < cnt; ++i) {
    float ms = 0.f;
    if (t->tmark[i] != t->tmark[i + 1]) {   // equal marks: the operator launched nothing
      hipError_t e = hipEventElapsedTime(&ms, t->tev[t->tmark[i]], t->tev[t->tmark[i + 1]]);
      if (e != hipSuccess) return fail(FP_ERR_DEVICE, "elapsed time: %s", hipGetErrorString(e));
    }
    ms_out[i] = ms;
  }
  *n_out = cnt;
  return FP_OK;
}

void fp_prefill_end(fp_prefill* t) {
  if (!t) return;
  fp_model* m = t->model;
  (void)hipStreamSynchronize(m->stream);
  release_workspace(m, t->ws);
  if (!t->owned_blocks.empty()) (void)fp_kv_free(m, (int32_t)t->owned_blocks.size(), t->owned_blocks.data());
  release_events(m, false, kMarkRing, t->ring);
  release_events(m, true, (int)t->tev.size(), t->tev.data());
  {
    std::lock_guard<std::mutex> lk(m->mu);
    m->live_tasks--;
  }
  delete t;
}

fp_status fp_prefill_moe_routing(fp_prefill* t, int32_t layer, int32_t* ids_out, float* weights_out) {
  if (!t || !ids_out || !weights_out) return fail(FP_ERR_INVALID, "fp_prefill_moe_routing: null argument");
  const fp_shape& sh = t->model->shape;
  if (sh.n_experts == 0) return fail(FP_ERR_INVALID, "fp_prefill_moe_routing: dense model");
  if (layer < 0 || layer >= sh.n_layers) return fail(FP_ERR_INVALID, "fp_prefill_moe_routing: layer out of range");
  int32_t cl = 0, co = 0;
  (void)fp_prefill_cursor(t, &cl, &co);
  if (cl * FP_OPS_PER_LAYER + co <= layer * FP_OPS_PER_LAYER + 6)
    return fail(FP_ERR_STATE, "fp_prefill_moe_routing: that layer's gate operator has not run yet");
  const size_t n = (size_t)t->n_tokens * sh.top_k;
  FP_HIP(hipStreamSynchronize(t->model->stream));
  if (n) {
    FP_HIP(hipMemcpy(ids_out, t->moe_ids + (size_t)layer * n, n * 4, hipMemcpyDeviceToDevice));
    FP_HIP(hipMemcpy(weights_out, t->moe_wts + (size_t)layer * n, n * 4, hipMemcpyDeviceToDevice));
  }
  return FP_OK;
}

fp_status fp_diag_mfma_ceiling(int32_t milliseconds, void* hip_stream, double* tflops_out) {
  if (!tflops_out || milliseconds <= 0 || milliseconds > 5000)
    return fail(FP_ERR_INVALID, "fp_diag_mfma_ceiling: milliseconds must be in 1..5000");
  hipStream_t s = reinterpret_cast<hipStream_t>(hip_stream);
  int cus = 0, dev = 0;
  FP_HIP(hipGetDevice(&dev));
  FP_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
  const int blocks = cus > 0 ? cus : 256;               // one workgroup of 8 waves per CU
  float* sink = nullptr;
  FP_HIP(hipMalloc(&sink, (size_t)blocks * 512 * sizeof(float)));
  hipEvent_t e0 = nullptr, e1 = nullptr;
  fp_status st = FP_OK;
  double best = 0.0;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) st = fail(FP_ERR_DEVICE, "event creation failed");
  // 20000 iterations of 8 MFMAs are ~2.7 ms at full rate; repeat until the time budget is used
  // (the clock settles under load) and report the last launch.
  const int iters = 20000;
  float total_ms = 0.f;
  (void)fp::launch_mfma_ceiling(sink, blocks, 100, s);  // warm-up
  while (st == FP_OK && total_ms < (float)milliseconds) {
    (void)hipEventRecord(e0, s);
    const double flops = fp::launch_mfma_ceiling(sink, blocks, iters, s);
    (void)hipEventRecord(e1, s);
    if (hipEventSynchronize(e1) != hipSuccess) { st = fail(FP_ERR_DEVICE, "mfma ceiling launch failed"); break; }
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    if (ms <= 0.f) { st = fail(FP_ERR_DEVICE, "mfma ceiling: no time measured"); break; }
    total_ms += ms;
    best = flops / (ms * 1e-3) / 1e12;
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(sink);
  if (st == FP_OK) *tflops_out = best;
  return st;
}

fp_status fp_op_gemm_ws(int32_t dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                        int64_t k, int32_t residual, void* workspace, int64_t workspace_bytes,
                        void* hip_stream) {
  if (!a || !w || !c || m <= 0 || n <= 0 || k <= 0 || (k % 8) || (n % 8) || m > INT32_MAX ||
      n > INT32_MAX || k > INT32_MAX || (dtype != 0 && dtype != 1))
    return fail(FP_ERR_INVALID, "fp_op_gemm: bad size, alignment or dtype");
  if (workspace_bytes < 0 || (workspace_bytes > 0 && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255))))
    return fail(FP_ERR_INVALID, "fp_op_gemm_ws: workspace null, misaligned (256 bytes) or negative size");
  fp::launch_gemm(dtype, a, w, c, m, n, k, residual, workspace, (size_t)workspace_bytes,
                  reinterpret_cast<hipStream_t>(hip_stream));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? FP_OK : fail(FP_ERR_DEVICE, "gemm launch: %s", hipGetErrorString(e));
}

fp_status fp_op_gemm(int32_t dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                     int64_t k, int32_t residual, void* hip_stream) {
  return fp_op_gemm_ws(dtype, a, w, c, m, n, k, residual, nullptr, 0, hip_stream);
}

fp_status fp_op_gemm_tail(int32_t dtype, const void* a, const void* w, void* c, int64_t m, int64_t n,
                          int64_t k, int32_t residual, void* workspace, int64_t workspace_bytes,
                          int32_t tail, const void* gain, void* tail_out, float eps, void* hip_stream) {
  if (!a || !w || m <= 0 || n <= 0 || k <= 0 || (k % 8) || (n % 8) || m > INT32_MAX || n > INT32_MAX ||
      k > INT32_MAX || dtype != FP_DTYPE_BF16 || !workspace || workspace_bytes <= 0 ||
      (reinterpret_cast<uintptr_t>(workspace) & 255) || !tail_out)
    return fail(FP_ERR_INVALID, "fp_op_gemm_tail: bad size, alignment, dtype or null buffer");
  const bool norm = tail == FP_TAIL_RMSNORM, swiglu = tail == FP_TAIL_SWIGLU;
  if (!(norm && residual && gain && c) && !(swiglu && !residual))
    return fail(FP_ERR_INVALID, "fp_op_gemm_tail: FP_TAIL_RMSNORM goes with residual = 1 (and gain, c), FP_TAIL_SWIGLU with residual = 0");
  const int kind = norm ? fp::kTailRmsNorm : fp::kTailSwiGLU;
  if (!fp::gemm_tail_fusable(dtype, m, n, k, (size_t)workspace_bytes, kind))
    return fail(FP_ERR_INVALID, "fp_op_gemm_tail: this problem is not cut over K with %lld bytes of workspace "
                                "(the tail rides on the split-K reduction); use the separate operators",
                (long long)workspace_bytes);
  const fp::GemmTail t{kind, gain, tail_out, eps};
  fp::launch_gemm(dtype, a, w, c, m, n, k, residual, workspace, (size_t)workspace_bytes,
                  reinterpret_cast<hipStream_t>(hip_stream), &t);
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? FP_OK : fail(FP_ERR_DEVICE, "gemm launch: %s", hipGetErrorString(e));
}

int64_t fp_op_gemm_workspace_bytes(int32_t dtype, int64_t m, int64_t n, int64_t k) {
  if (m <= 0 || n <= 0 || k <= 0) return 0;
  return (int64_t)fp::gemm_workspace_bytes(dtype, m, n, k);
}

fp_status fp_op_gemm_swiglu(const void* a, const void* w_gate_up, void* out, int64_t m, int64_t f,
                            int64_t k, void* hip_stream) {
  if (!a || !w_gate_up || !out || m <= 0 || f <= 0 || k <= 0 || m > INT32_MAX || 2 * f > INT32_MAX ||
      k > INT32_MAX)
    return fail(FP_ERR_INVALID, "fp_op_gemm_swiglu: bad size");
  if (!fp::gemm_swiglu_fusable(FP_DTYPE_BF16, m, f, k))
    return fail(FP_ERR_INVALID, "fp_op_gemm_swiglu: shape not handled by the fused kernel "
                                "(needs K %% 64 == 0, F %% 8 == 0 and at least 96 output tiles)");
  fp::launch_gemm_swiglu(a, w_gate_up, out, m, f, k, reinterpret_cast<hipStream_t>(hip_stream));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? FP_OK : fail(FP_ERR_DEVICE, "gemm_swiglu launch: %s", hipGetErrorString(e));
}

fp_status fp_op_rmsnorm(int32_t dtype, const void* x_f32, const void* gain, void* out, int64_t t,
                        int64_t d, float eps, void* hip_stream) {
  if (!x_f32 || !gain || !out || t <= 0 || d <= 0 || (d % 8) || (dtype != 0 && dtype != 1))
    return fail(FP_ERR_INVALID, "fp_op_rmsnorm: bad size or dtype");
  fp::launch_rmsnorm(dtype, (const float*)x_f32, gain, out, t, d, eps, reinterpret_cast<hipStream_t>(hip_stream));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? FP_OK : fail(FP_ERR_DEVICE, "rmsnorm launch: %s", hipGetErrorString(e));
}

fp_status fp_op_silu_mul(int32_t dtype, const void* gu, void* out, int64_t t, int64_t f,
                         void* hip_stream) {
  if (!gu || !out || t <= 0 || f <= 0 || (f % 8) || (dtype != 0 && dtype != 1))
    return fail(FP_ERR_INVALID, "fp_op_silu_mul: bad size or dtype");
  fp::launch_silu_mul(dtype, gu, out, t, f, reinterpret_cast<hipStream_t>(hip_stream));
  hipError_t e = hipGetLastError();
  return e == hipSuccess ? FP_OK : fail(FP_ERR_DEVICE, "silu_mul launch: %s", hipGetErrorString(e));
}

}  // extern "C"
