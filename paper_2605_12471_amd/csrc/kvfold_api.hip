// Host side of libkvfold: the C ABI declared in include/kvfold.h.
//
// One fold step (paper Sec. 2, "KV-Fold" and "A recurrent view") = validate positions, enqueue
// the append of the chunk's K/V rows (its own kernel, or part of the attention kernel), enqueue
// chunk-prefix attention over rows [0, len + C), and, when the key range was split over workgroups,
// enqueue the merge.  Everything is stream-ordered;
// nothing here synchronises or allocates after kvfold_cache_create.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/kvfold.h"
#include "kvfold_host.h"
#include "kvfold_internal.h"

using namespace kvfold;

struct kvfold_cache {
  PlanCtx pc;  // configuration, workspace size, CU count, tuning knobs, storage round trip: what the planner reads
  int elem_bytes;
  float scale;
  unsigned char* kv;  // K block then V block, each [layer][Hkv][cap][d]
  bool owns_kv;
  size_t kv_bytes;
  float* ws_o;   // split workspace: unnormalised partial outputs
  float* ws_ml;  // split workspace: (max, sum) pairs
  std::vector<int64_t> len;
  // optional per-kernel timing: 4 events per step (before append, after append, after attention, after merge)
  std::vector<hipEvent_t> prof_events;
  std::vector<char> prof_has_merge;
  int prof_max_steps = 0;
  int prof_steps = 0;
};

namespace {
thread_local int g_last_hip_error = 0;
}

namespace kvfold {
int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  (void)hipGetLastError();  // clear the sticky error
  return e == hipErrorOutOfMemory ? KVFOLD_ERR_OOM : KVFOLD_ERR_HIP;
}
}  // namespace kvfold

namespace {

// ---- static scratch of kvfold_step_noalloc: split partials for callers that cannot allocate ------------
// One array per GPU, part of the library's code object, alive until the process ends.  Holds the (max, sum)
// pairs of kStaticScratchRows (row, split) pairs first, then their unnormalised partial outputs (head_dim
// floats each, 128 at most).  Host code never uses the symbol itself as an address: the per-device pointer
// comes from hipGetSymbolAddress, once per device.
constexpr int64_t kStaticScratchRows = 1 << 17;                                    // (row, split) pairs
constexpr size_t kStaticScratchBytes = (size_t)kStaticScratchRows * (128 + 2) * sizeof(float);  // 65 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
unsigned char* g_scratch_ptr[kMaxDevices] = {};

// Device address of this device's copy of the scratch array (the device must be current).
int static_scratch(int device, unsigned char** out) {
  if (device < 0 || device >= kMaxDevices) return KVFOLD_ERR_INVALID_ARG;
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_fail(e);
    if (!ptr) return KVFOLD_ERR_HIP;
    g_scratch_ptr[device] = static_cast<unsigned char*>(ptr);
  }
  *out = g_scratch_ptr[device];
  return KVFOLD_OK;
}

struct DeviceGuard {
  int prev = -1;
  bool switched = false;
  hipError_t err = hipSuccess;
  explicit DeviceGuard(int dev) {
    err = hipGetDevice(&prev);
    if (err == hipSuccess && prev != dev) {
      err = hipSetDevice(dev);
      switched = (err == hipSuccess);
    }
  }
  ~DeviceGuard() {
    if (switched) (void)hipSetDevice(prev);
  }
};

}  // namespace

extern "C" {

int kvfold_cache_create(const kvfold_config_t* cfg, kvfold_cache_t** out_cache) {
  if (out_cache) *out_cache = nullptr;
  if (!out_cache) return KVFOLD_ERR_INVALID_ARG;
  int rc = validate_config(cfg);
  if (rc != KVFOLD_OK) return rc;
  const size_t need = bytes_required(cfg);
  if (cfg->kv_buffer && cfg->kv_buffer_bytes < need) return KVFOLD_ERR_OOM;

  int n_dev = 0;
  hipError_t e = hipGetDeviceCount(&n_dev);
  if (e != hipSuccess) return hip_fail(e);
  if (cfg->device >= n_dev || cfg->device >= kMaxDevices) return KVFOLD_ERR_INVALID_ARG;
  DeviceGuard guard(cfg->device);
  if (guard.err != hipSuccess) return hip_fail(guard.err);

  kvfold_cache* c = new (std::nothrow) kvfold_cache();
  if (!c) return KVFOLD_ERR_OOM;
  c->pc = PlanCtx{};
  c->pc.cfg = *cfg;
  c->elem_bytes = elem_size(cfg->dtype);
  c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  c->kv = nullptr;
  c->owns_kv = false;
  c->kv_bytes = need;
  c->ws_o = nullptr;
  c->ws_ml = nullptr;
  c->len.assign((size_t)cfg->n_layers, 0);

  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, cfg->device);
  // whatever a launch could still refuse (the attention kernels' LDS size) is settled here, so that a step
  // never fails with part of its work already on the stream
  if (e == hipSuccess && cfg->dtype == KVFOLD_BF16) e = prepare_attn_bf16(cfg->head_dim);
  unsigned char* scratch_ptr = nullptr;
  if (e == hipSuccess && static_scratch(cfg->device, &scratch_ptr) != KVFOLD_OK) e = hipErrorInvalidSymbol;
  if (e != hipSuccess) {
    delete c;
    return hip_fail(e);
  }
  c->pc.n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

  if (cfg->kv_buffer) {
    c->kv = static_cast<unsigned char*>(cfg->kv_buffer);
  } else {
    void* ptr = nullptr;
    e = hipMalloc(&ptr, need);
    if (e != hipSuccess) {
      delete c;
      return hip_fail(e);
    }
    c->kv = static_cast<unsigned char*>(ptr);
    c->owns_kv = true;
  }

  const int64_t ws_rows = workspace_rows(cfg);
  if (ws_rows > 0) {
    void *po = nullptr, *pm = nullptr;
    e = hipMalloc(&po, (size_t)ws_rows * cfg->head_dim * sizeof(float));
    if (e == hipSuccess) e = hipMalloc(&pm, (size_t)ws_rows * 2 * sizeof(float));
    if (e != hipSuccess) {
      if (po) (void)hipFree(po);
      if (c->owns_kv) (void)hipFree(c->kv);
      delete c;
      return hip_fail(e);
    }
    c->ws_o = static_cast<float*>(po);
    c->ws_ml = static_cast<float*>(pm);
    c->pc.ws_rows = ws_rows;
  }
  *out_cache = c;
  return KVFOLD_OK;
}

}  // extern "C"

namespace {

struct StepOpts {
  const float* rope_cos = nullptr;  // both null (inputs used as handed in) or both set
  const float* rope_sin = nullptr;
  int32_t n_sink = 0;               // sink + sliding-window step when window > 0
  int64_t window = 0;
  bool static_scratch = false;      // split partials go to the library's static array instead of the cache's workspace
};

// One fold step.
int step_impl(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new, int32_t n_tokens,
              int64_t pos_offset, const StepOpts& opt, void* out, float* lse, void* stream) {
  if (!c || !q || !k_new || !v_new || !out) return KVFOLD_ERR_INVALID_ARG;
  const kvfold_config_t& f = c->pc.cfg;
  if (layer < 0 || layer >= f.n_layers) return KVFOLD_ERR_BAD_LAYER;
  if (n_tokens < 1 || n_tokens > f.chunk_tokens) return KVFOLD_ERR_INVALID_ARG;
  const int64_t len_prev = c->len[(size_t)layer];
  if (pos_offset != len_prev) return KVFOLD_ERR_POSITION;
  if (len_prev + n_tokens > f.capacity_tokens) return KVFOLD_ERR_CAPACITY;
  if ((reinterpret_cast<uintptr_t>(q) | reinterpret_cast<uintptr_t>(k_new) | reinterpret_cast<uintptr_t>(v_new) |
       reinterpret_cast<uintptr_t>(out)) & 15)
    return KVFOLD_ERR_INVALID_ARG;  // the kernels move 16-byte vectors

  DeviceGuard guard(f.device);
  if (guard.err != hipSuccess) return hip_fail(guard.err);
  hipStream_t s = static_cast<hipStream_t>(stream);

  // where the split partials go, and how many (row, split) pairs fit there
  PlanCtx pc = c->pc;
  float *part_o = c->ws_o, *part_ml = c->ws_ml;
  if (opt.static_scratch) {
    unsigned char* sp = nullptr;
    const int rc = static_scratch(f.device, &sp);
    if (rc != KVFOLD_OK) return rc;
    const int64_t rows = (int64_t)n_tokens * f.n_q_heads;
    if (2 * rows > kStaticScratchRows) return KVFOLD_ERR_SCRATCH;  // not even two pieces of this step fit
    pc.ws_rows = kStaticScratchRows;
    part_ml = reinterpret_cast<float*>(sp);
    part_o = reinterpret_cast<float*>(sp + (size_t)kStaticScratchRows * 2 * sizeof(float));
  }

  const size_t layer_block = (size_t)f.n_kv_heads * (size_t)f.capacity_tokens * (size_t)f.head_dim * c->elem_bytes;
  unsigned char* k_layer = c->kv + (size_t)layer * layer_block;
  unsigned char* v_layer = c->kv + c->kv_bytes / 2 + (size_t)layer * layer_block;

  AppendParams ap;
  ap.k_new = k_new;
  ap.v_new = v_new;
  ap.k_cache = k_layer;
  ap.v_cache = v_layer;
  ap.n_tokens = n_tokens;
  ap.n_kv_heads = f.n_kv_heads;
  ap.row_bytes = f.head_dim * c->elem_bytes;
  ap.capacity = f.capacity_tokens;
  ap.len_prev = len_prev;
  ap.rope_cos = opt.rope_cos;
  ap.rope_sin = opt.rope_sin;
  ap.elem_is_bf16 = f.dtype == KVFOLD_BF16;

  const Plan pl = make_plan(pc, n_tokens, len_prev + n_tokens, opt.n_sink, opt.window);
  AttnParams at;
  at.q = q;
  at.k_cache = k_layer;
  at.v_cache = v_layer;
  at.out = out;
  at.lse = lse;
  at.part_o = part_o;
  at.part_ml = part_ml;
  at.n_tokens = n_tokens;
  at.n_q_heads = f.n_q_heads;
  at.n_kv_heads = f.n_kv_heads;
  at.group = f.n_q_heads / f.n_kv_heads;
  at.capacity = f.capacity_tokens;
  at.len_prev = len_prev;
  at.n_splits = pl.n_splits;
  at.tiles_per_split = pl.tiles_per_split;
  at.units_per_head = pl.units_per_head;
  at.wgs_per_head = pl.wgs_per_head;
  at.n_wgs = pl.n_wgs;
  at.pair_order = pl.pair_order;
  at.pair_units = pl.pair_units;
  at.scale_log2e = c->scale * 1.4426950408889634f;
  at.rope_cos = opt.rope_cos;
  at.rope_sin = opt.rope_sin;
  at.n_sink = opt.n_sink;
  at.window = (int32_t)opt.window;
  // The bf16 attention kernel appends by itself when the cache length is a whole number of key tiles (every
  // chunk length that is a multiple of 64), nothing has to happen to the rows on their way in, and the chunk's
  // rows can be addressed with 32-bit byte offsets.
  const bool fused_append = fused_append_applies(pc, n_tokens, len_prev, opt.rope_cos != nullptr);
  at.k_new = fused_append ? k_new : nullptr;
  at.v_new = fused_append ? v_new : nullptr;
  if (pl.n_splits > 1 && ((int64_t)pl.n_splits * n_tokens * f.n_q_heads > pc.ws_rows || !part_o))
    return KVFOLD_ERR_HIP;  // planner bug guard

  hipEvent_t* ev = nullptr;
  if (c->prof_max_steps > 0 && c->prof_steps < c->prof_max_steps) ev = &c->prof_events[(size_t)c->prof_steps * 4];
  hipError_t e = hipSuccess;
  if (ev) {
    e = hipEventRecord(ev[0], s);
    if (e != hipSuccess) return hip_fail(e);
  }
  if (!fused_append) {
    e = launch_append(ap, s);
    if (e != hipSuccess) return hip_fail(e);
  }
  if (pc.storage_bits) {
    e = launch_storage_roundtrip(ap, pc.storage_bits, s);
    if (e != hipSuccess) return hip_fail(e);
  }
  const bool own_append = !fused_append || pc.storage_bits;  // something ran between ev[0] and the attention kernel
  if (ev && own_append) (void)hipEventRecord(ev[1], s);
  e = (f.dtype == KVFOLD_BF16) ? launch_attn_bf16(at, f.head_dim, pl.units_per_wave, s) : launch_attn_f32(at, f.head_dim, s);
  if (e != hipSuccess) return hip_fail(e);
  if (ev) (void)hipEventRecord(ev[2], s);
  if (pl.n_splits > 1) {
    CombineParams cp;
    cp.part_o = part_o;
    cp.part_ml = part_ml;
    cp.out = out;
    cp.lse = lse;
    cp.n_rows = n_tokens * f.n_q_heads;
    cp.n_tokens = n_tokens;
    cp.n_q_heads = f.n_q_heads;
    cp.head_dim = f.head_dim;
    cp.n_splits = pl.n_splits;
    cp.out_is_bf16 = f.dtype == KVFOLD_BF16;
    e = launch_combine(cp, s);
    if (e != hipSuccess) return hip_fail(e);
  }
  if (ev) {
    if (pl.n_splits > 1) (void)hipEventRecord(ev[3], s);
    c->prof_has_merge[(size_t)c->prof_steps] = (char)((pl.n_splits > 1 ? 1 : 0) | (own_append ? 2 : 0));
    c->prof_steps++;
  }
  c->len[(size_t)layer] = len_prev + n_tokens;
  return KVFOLD_OK;
}

}  // namespace

extern "C" {

int kvfold_step_ex(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new,
                   int32_t n_tokens, int64_t pos_offset, void* out, float* lse, void* stream) {
  return step_impl(c, layer, q, k_new, v_new, n_tokens, pos_offset, StepOpts{}, out, lse, stream);
}

int kvfold_step_rope(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new,
                     int32_t n_tokens, int64_t pos_offset, const float* rope_cos, const float* rope_sin, void* out,
                     float* lse, void* stream) {
  if (!rope_cos || !rope_sin) return KVFOLD_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(rope_cos) | reinterpret_cast<uintptr_t>(rope_sin)) & 15) return KVFOLD_ERR_INVALID_ARG;
  StepOpts opt;
  opt.rope_cos = rope_cos;
  opt.rope_sin = rope_sin;
  return step_impl(c, layer, q, k_new, v_new, n_tokens, pos_offset, opt, out, lse, stream);
}

int kvfold_step_window(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new,
                       int32_t n_tokens, int64_t pos_offset, int32_t n_sink, int64_t window, void* out, float* lse,
                       void* stream) {
  if (n_sink < 0 || window < 1 || window > ((int64_t)1 << 30)) return KVFOLD_ERR_INVALID_ARG;
  StepOpts opt;
  opt.n_sink = n_sink;
  opt.window = window;
  return step_impl(c, layer, q, k_new, v_new, n_tokens, pos_offset, opt, out, lse, stream);
}

int kvfold_step_noalloc(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new,
                        int32_t n_tokens, int64_t pos_offset, void* out, float* lse, void* stream) {
  StepOpts opt;
  opt.static_scratch = true;
  return step_impl(c, layer, q, k_new, v_new, n_tokens, pos_offset, opt, out, lse, stream);
}

int kvfold_step(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new, int64_t pos_offset,
                void* out, void* stream) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  return kvfold_step_ex(c, layer, q, k_new, v_new, c->pc.cfg.chunk_tokens, pos_offset, out, nullptr, stream);
}

int kvfold_cache_destroy(kvfold_cache_t* c) {
  if (!c) return KVFOLD_OK;
  int rc = KVFOLD_OK;
  {
    DeviceGuard guard(c->pc.cfg.device);
    if (guard.err != hipSuccess) rc = hip_fail(guard.err);
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) rc = hip_fail(e);
    for (auto& x : c->prof_events)
      if (x) (void)hipEventDestroy(x);
    if (c->owns_kv && c->kv) (void)hipFree(c->kv);
    if (c->ws_o) (void)hipFree(c->ws_o);
    if (c->ws_ml) (void)hipFree(c->ws_ml);
  }
  delete c;
  return rc;
}

int64_t kvfold_cache_length(const kvfold_cache_t* c, int layer) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  if (layer < 0 || layer >= c->pc.cfg.n_layers) return KVFOLD_ERR_BAD_LAYER;
  return c->len[(size_t)layer];
}

int kvfold_cache_view(const kvfold_cache_t* c, int layer, void** k_dev, void** v_dev, int64_t* row_stride_elems,
                      int64_t* head_stride_elems) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  const kvfold_config_t& f = c->pc.cfg;
  if (layer < 0 || layer >= f.n_layers) return KVFOLD_ERR_BAD_LAYER;
  const size_t layer_block = (size_t)f.n_kv_heads * (size_t)f.capacity_tokens * (size_t)f.head_dim * c->elem_bytes;
  if (k_dev) *k_dev = c->kv + (size_t)layer * layer_block;
  if (v_dev) *v_dev = c->kv + c->kv_bytes / 2 + (size_t)layer * layer_block;
  if (row_stride_elems) *row_stride_elems = f.head_dim;
  if (head_stride_elems) *head_stride_elems = f.capacity_tokens * f.head_dim;
  return KVFOLD_OK;
}

int kvfold_cache_truncate(kvfold_cache_t* c, int layer, int64_t new_len) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  if (layer < -1 || layer >= c->pc.cfg.n_layers) return KVFOLD_ERR_BAD_LAYER;
  if (new_len < 0) return KVFOLD_ERR_INVALID_ARG;
  if (layer == -1) {
    for (int64_t v : c->len)
      if (new_len > v) return KVFOLD_ERR_POSITION;
    for (auto& v : c->len) v = new_len;
  } else {
    if (new_len > c->len[(size_t)layer]) return KVFOLD_ERR_POSITION;
    c->len[(size_t)layer] = new_len;
  }
  return KVFOLD_OK;
}

int kvfold_cache_set_length(kvfold_cache_t* c, int layer, int64_t new_len) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  if (layer < -1 || layer >= c->pc.cfg.n_layers) return KVFOLD_ERR_BAD_LAYER;
  if (new_len < 0) return KVFOLD_ERR_INVALID_ARG;
  if (new_len > c->pc.cfg.capacity_tokens) return KVFOLD_ERR_CAPACITY;
  if (layer == -1)
    for (auto& v : c->len) v = new_len;
  else
    c->len[(size_t)layer] = new_len;
  return KVFOLD_OK;
}

int kvfold_cache_set_storage_roundtrip(kvfold_cache_t* c, int32_t n_bits) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  if (n_bits != 0 && n_bits != 4 && n_bits != 8) return KVFOLD_ERR_INVALID_ARG;
  if (n_bits != 0 && c->pc.cfg.dtype != KVFOLD_BF16) return KVFOLD_ERR_UNSUPPORTED;
  c->pc.storage_bits = n_bits;
  return KVFOLD_OK;
}

int kvfold_cache_set_tuning(kvfold_cache_t* c, int32_t knob, int32_t value) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  switch (knob) {
    case KVFOLD_TUNE_SPLITS:
      if (value < 0 || value > kMaxSplits) return KVFOLD_ERR_INVALID_ARG;
      c->pc.tune_splits = value;
      return KVFOLD_OK;
    case KVFOLD_TUNE_PAIR_UNITS:
      if (value < 0 || value > 2) return KVFOLD_ERR_INVALID_ARG;
      c->pc.tune_pair_units = value;
      return KVFOLD_OK;
    case KVFOLD_TUNE_FUSED_APPEND:
      if (value < 0 || value > 1) return KVFOLD_ERR_INVALID_ARG;
      c->pc.tune_fused_append = value;
      return KVFOLD_OK;
    case KVFOLD_TUNE_UNITS_PER_WAVE:
      if (value < 0 || value > 2) return KVFOLD_ERR_INVALID_ARG;
      c->pc.tune_units_per_wave = value;
      return KVFOLD_OK;
    default:
      return KVFOLD_ERR_INVALID_ARG;
  }
}

int kvfold_cache_plan(const kvfold_cache_t* c, int32_t n_tokens, int64_t len_after, int32_t* n_workgroups,
                      int32_t* n_splits) {
  if (!c || n_tokens < 1 || n_tokens > c->pc.cfg.chunk_tokens || len_after < n_tokens ||
      len_after > c->pc.cfg.capacity_tokens)
    return KVFOLD_ERR_INVALID_ARG;
  const Plan pl = make_plan(c->pc, n_tokens, len_after, 0, 0);
  if (n_workgroups) *n_workgroups = pl.n_wgs;
  if (n_splits) *n_splits = pl.n_splits;
  return KVFOLD_OK;
}

int kvfold_cache_profile_begin(kvfold_cache_t* c, int32_t max_steps) {
  if (!c || max_steps < 1 || max_steps > (1 << 20) || c->prof_max_steps > 0) return KVFOLD_ERR_INVALID_ARG;
  DeviceGuard guard(c->pc.cfg.device);
  if (guard.err != hipSuccess) return hip_fail(guard.err);
  c->prof_events.assign((size_t)max_steps * 4, nullptr);
  for (auto& ev : c->prof_events) {
    hipError_t e = hipEventCreate(&ev);
    if (e != hipSuccess) {
      for (auto& x : c->prof_events)
        if (x) (void)hipEventDestroy(x);
      c->prof_events.clear();
      return hip_fail(e);
    }
  }
  c->prof_has_merge.assign((size_t)max_steps, 0);
  c->prof_max_steps = max_steps;
  c->prof_steps = 0;
  return KVFOLD_OK;
}

int kvfold_cache_profile_end(kvfold_cache_t* c, int32_t* n_steps, double* append_ms, double* attention_ms,
                             double* merge_ms) {
  if (!c || c->prof_max_steps == 0) return KVFOLD_ERR_INVALID_ARG;
  DeviceGuard guard(c->pc.cfg.device);
  int rc = KVFOLD_OK;
  hipError_t e = hipDeviceSynchronize();
  if (e != hipSuccess) rc = hip_fail(e);
  double a = 0, t = 0, m = 0;
  for (int i = 0; i < c->prof_steps && rc == KVFOLD_OK; ++i) {
    hipEvent_t* ev = &c->prof_events[(size_t)i * 4];
    float ms = 0.f;
    const int flags = c->prof_has_merge[(size_t)i];  // bit 0: a merge kernel ran, bit 1: the append ran as its own kernel
    if (flags & 2) {
      if (hipEventElapsedTime(&ms, ev[0], ev[1]) == hipSuccess) a += ms;
      if (hipEventElapsedTime(&ms, ev[1], ev[2]) == hipSuccess) t += ms;
    } else if (hipEventElapsedTime(&ms, ev[0], ev[2]) == hipSuccess) {
      t += ms;  // the attention kernel appended by itself
    }
    if ((flags & 1) && hipEventElapsedTime(&ms, ev[2], ev[3]) == hipSuccess) m += ms;
  }
  if (n_steps) *n_steps = c->prof_steps;
  if (append_ms) *append_ms = a;
  if (attention_ms) *attention_ms = t;
  if (merge_ms) *merge_ms = m;
  for (auto& x : c->prof_events)
    if (x) (void)hipEventDestroy(x);
  c->prof_events.clear();
  c->prof_has_merge.clear();
  c->prof_max_steps = 0;
  c->prof_steps = 0;
  return rc;
}

int kvfold_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
