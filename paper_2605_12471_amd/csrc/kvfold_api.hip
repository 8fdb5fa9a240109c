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
#include "kvfold_internal.h"

using namespace kvfold;

struct kvfold_cache {
  kvfold_config_t cfg;
  int elem_bytes;
  float scale;
  unsigned char* kv;  // K block then V block, each [layer][Hkv][cap][d]
  bool owns_kv;
  size_t kv_bytes;
  float* ws_o;   // split workspace: unnormalised partial outputs
  float* ws_ml;  // split workspace: (max, sum) pairs
  int64_t ws_rows;
  int n_cu;
  std::vector<int64_t> len;
  int tune_splits;
  int tune_units_per_wave;
  int tune_pair_units;  // 0 automatic, 1 never, 2 whenever the two-unit kernel runs
  int tune_fused_append;  // 0 automatic (whenever possible), 1 never: always the separate append kernel
  int storage_bits;  // 0, or 4 / 8: rows are round-tripped through that integer width as they join the cache
  // optional per-kernel timing: 4 events per step (before append, after append, after attention, after merge)
  std::vector<hipEvent_t> prof_events;
  std::vector<char> prof_has_merge;
  int prof_max_steps = 0;
  int prof_steps = 0;
};

namespace {

thread_local int g_last_hip_error = 0;

int hip_fail(hipError_t e) {
  g_last_hip_error = (int)e;
  (void)hipGetLastError();  // clear the sticky error
  return e == hipErrorOutOfMemory ? KVFOLD_ERR_OOM : KVFOLD_ERR_HIP;
}

int elem_size(int dtype) { return dtype == KVFOLD_F32 ? 4 : dtype == KVFOLD_BF16 ? 2 : 0; }

int validate_config(const kvfold_config_t* c) {
  if (!c || c->struct_size != sizeof(kvfold_config_t)) return KVFOLD_ERR_INVALID_ARG;
  if (c->n_layers < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->chunk_tokens < 1 || c->capacity_tokens < 1 ||
      c->device < 0 || !(c->softmax_scale >= 0.f) || !std::isfinite(c->softmax_scale))
    return KVFOLD_ERR_INVALID_ARG;
  if (c->kv_buffer && (reinterpret_cast<uintptr_t>(c->kv_buffer) & 255)) return KVFOLD_ERR_INVALID_ARG;
  if (elem_size(c->dtype) == 0) return KVFOLD_ERR_UNSUPPORTED;
  if (c->head_dim != 64 && c->head_dim != 128) return KVFOLD_ERR_UNSUPPORTED;
  if (c->n_q_heads % c->n_kv_heads) return KVFOLD_ERR_UNSUPPORTED;
  // sizes the kernels index with 32-bit row counts / 64-bit byte offsets
  if (c->capacity_tokens > (int64_t)1 << 30 || (int64_t)c->chunk_tokens * c->n_q_heads > (int64_t)1 << 28)
    return KVFOLD_ERR_UNSUPPORTED;
  // the attention kernels address one KV head's rows with 32-bit byte offsets
  if (c->capacity_tokens * c->head_dim * elem_size(c->dtype) > (int64_t)0xFFFFFFFFll) return KVFOLD_ERR_UNSUPPORTED;
  if (c->chunk_tokens > c->capacity_tokens) return KVFOLD_ERR_INVALID_ARG;
  return KVFOLD_OK;
}

size_t bytes_required(const kvfold_config_t* c) {
  return (size_t)c->n_layers * 2u * (size_t)c->n_kv_heads * (size_t)c->capacity_tokens * (size_t)c->head_dim *
         (size_t)elem_size(c->dtype);
}

constexpr int64_t kMaxSplitRows = 1 << 19;  // cap on S * C * Hq rows held in the split workspace
constexpr int kMaxSplits = 64;
constexpr int kMinTilesPerSplit = 8;

struct Plan {
  int units_per_wave, units_per_head, wgs_per_head, n_splits, tiles_per_split, n_wgs, pair_order, pair_units;
};

// Launch geometry for `upw` units per wavefront: enough prefix splits to put at least `target`
// workgroups on the chip when the unsplit grid has fewer (a forced split count overrides that).
Plan plan_with(const kvfold_cache* c, int n_tokens, int64_t len_after, int upw) {
  const kvfold_config_t& f = c->cfg;
  const int G = f.n_q_heads / f.n_kv_heads;
  Plan pl;
  pl.pair_order = 0;
  pl.pair_units = 0;
  pl.units_per_head = G * ((n_tokens + kRowsPerUnit - 1) / kRowsPerUnit);
  pl.units_per_wave = upw;
  const int per_wg = kUnitsPerWg * upw;
  pl.wgs_per_head = (pl.units_per_head + per_wg - 1) / per_wg;
  const int64_t base = (int64_t)f.n_kv_heads * pl.wgs_per_head;
  const int ntiles = (int)((len_after + kTileKeys - 1) / kTileKeys);
  int64_t s_max = c->tune_splits > 0 ? ntiles : ntiles / kMinTilesPerSplit;  // a forced count only needs a tile each
  const int64_t rows = (int64_t)n_tokens * f.n_q_heads;
  if (c->ws_rows / rows < s_max) s_max = c->ws_rows / rows;
  if (s_max > kMaxSplits) s_max = kMaxSplits;
  if (s_max < 1) s_max = 1;
  int64_t s = 1;
  if (c->tune_splits > 0) {
    s = c->tune_splits;
  } else {
    // Estimated time of the step for every split count; the smallest wins (by more than 0.5 %).
    //  * Attention itself at the rate of a full chip (1.35 PFLOP/s, or 5 TB/s for the K and V rows when that
    //    is longer), divided by what a partly filled last round still delivers.  The chip is power-limited:
    //    idle CUs hand their share to the busy ones, so 87.5 % of the CUs give 96 % of the rate (measured:
    //    rate ~ fill^0.3), until the busy CUs reach their top clock (1.41 x the full-chip clock).
    //  * Unsplit, several rounds, heaviest workgroups first: the slots left over in the last round idle for
    //    the length of the lightest workgroups only (first token block: the prefix and little else).
    //  * A residue of imbalance that more rounds even out, 8 us of start and end per round of workgroups,
    //    and for s > 1 the fp32 partials written and read once at 4 TB/s plus the combine launch.
    const int64_t slots = (int64_t)c->n_cu * (upw == 1 ? 2 : 1);
    const double flops = 4.0 * f.n_q_heads * f.head_dim * (double)n_tokens * ((double)len_after - 0.5 * n_tokens);
    const double kv_bytes = 2.0 * f.n_kv_heads * f.head_dim * (double)elem_size(f.dtype) * (double)len_after;
    const double t_attn = std::max(flops / (f.dtype == KVFOLD_BF16 ? 1.35e15 : 1.2e14), kv_bytes / 5e12);  // bf16 / fp32 MFMA rates
    double best = 1e30;
    for (int64_t cand = 1; cand <= s_max; ++cand) {
      // only split counts that whole tiles can realise; the last piece may be shorter than the others, and the
      // launch lasts as long as the longest
      const int64_t tps = (ntiles + cand - 1) / cand;
      if ((ntiles + tps - 1) / tps != cand) continue;
      const double uneven = (double)(tps * cand) / (double)ntiles;
      const int64_t w = base * cand, rounds = (w + slots - 1) / slots;
      double fill = (double)w / (double)(rounds * slots);
      if (cand == 1 && rounds >= 2) {
        const double w_min = (double)(len_after - n_tokens) + kRowsPerUnit, w_mean = (double)len_after - 0.5 * n_tokens;
        fill = (double)w * w_mean / ((double)w * w_mean + (double)(rounds * slots - w) * w_min);
      }
      const double rate = std::min(1.41 * fill, std::pow(fill, 0.3));
      const double merge = cand > 1 ? (double)cand * rows * (f.head_dim + 2) * 8.0 / 4e12 + 6e-6 : 0.0;
      const double t = t_attn * uneven / rate * (1.0 + 0.03 / (double)rounds) + 8e-6 * (double)rounds + merge;
      if (t < best * 0.995) {
        best = t;
        s = cand;
      }
    }
  }
  if (s > s_max) s = s_max;
  pl.tiles_per_split = (int)((ntiles + s - 1) / s);
  if (pl.tiles_per_split < 1) pl.tiles_per_split = 1;
  pl.n_splits = (ntiles + pl.tiles_per_split - 1) / pl.tiles_per_split;
  if (pl.n_splits < 1) pl.n_splits = 1;
  pl.n_wgs = (int)(base * pl.n_splits);
  return pl;
}

Plan choose_plan(const kvfold_cache* c, int n_tokens, int64_t len_after);

// split workspace: room for kMaxSplits pieces of one chunk, capped
int64_t workspace_rows(const kvfold_config_t* cfg) {
  const int64_t rows = (int64_t)cfg->chunk_tokens * cfg->n_q_heads;
  int64_t ws_rows = rows * kMaxSplits;
  if (ws_rows > kMaxSplitRows) ws_rows = kMaxSplitRows;
  if (ws_rows < 2 * rows) ws_rows = 0;  // chunks this large never need a split
  return ws_rows;
}

Plan make_plan(const kvfold_cache* c, int n_tokens, int64_t len_after) {
  Plan pl = choose_plan(c, n_tokens, len_after);
  // Two-unit kernel, a single round of workgroups: the causal part makes the last token block's wavefronts
  // longer than the first's (100 % on an empty cache, 6 % after 8 chunks) and nothing evens that out; pair
  // an early and a late row block in every wavefront instead (the late one finishes alone, at the
  // efficiency of a one-unit step).  Measured: +7 % down to +0.5 % at 31 chunks of prefix, even at 63; with
  // a split prefix (only the last pieces hold the causal part) +0.5 to 2 %, never a loss.  With several
  // rounds the dispatcher balances heaviest-first workgroups by itself and pairing only costs.
  if (c->cfg.dtype == KVFOLD_BF16 && pl.units_per_wave == 2 && c->tune_pair_units != 1) {
    if (c->tune_pair_units == 2 || pl.n_wgs <= c->n_cu) pl.pair_units = 1;
  }
  return pl;
}

Plan choose_plan(const kvfold_cache* c, int n_tokens, int64_t len_after) {
  const kvfold_config_t& f = c->cfg;
  if (f.dtype != KVFOLD_BF16) return plan_with(c, n_tokens, len_after, 1);
  if (c->tune_units_per_wave) return plan_with(c, n_tokens, len_after, c->tune_units_per_wave);
  Plan p1 = plan_with(c, n_tokens, len_after, 1);
  // Prefix shorter than the chunk: the causal part makes late token blocks several times as long as early
  // ones.  If the one-unit-per-wavefront grid is resident at once (two workgroups per CU), pair heavy with
  // light workgroups on a CU (measured faster than pairing units inside the two-unit kernel only here).
  const int64_t wgs1 = (int64_t)f.n_kv_heads * p1.wgs_per_head;
  if (c->tune_splits == 0 && len_after < 2 * (int64_t)n_tokens && wgs1 <= 2 * (int64_t)c->n_cu &&
      wgs1 > (int64_t)c->n_cu && p1.n_splits == 1) {
    p1.pair_order = 1;
    return p1;
  }
  // Two units per wavefront is the faster kernel (every LDS fragment feeds two MFMAs) whenever it
  // can fill the chip, if need be by splitting the prefix; one unit per wavefront is for grids too
  // small for that, and for chunks so short that half of the two-unit workgroup would idle.
  const Plan p2 = plan_with(c, n_tokens, len_after, 2);
  const int64_t padded1 = (int64_t)p1.wgs_per_head * kUnitsPerWg, padded2 = (int64_t)p2.wgs_per_head * kUnitsPerWg * 2;
  if (padded2 * 5 > padded1 * 6) return p1;                                   // more than 20 % extra padding
  if ((int64_t)p2.n_wgs * 4 < (int64_t)c->n_cu * 3 && p1.n_wgs > p2.n_wgs) return p1;  // cannot fill the chip
  return p2;
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

size_t kvfold_cache_bytes_required(const kvfold_config_t* cfg) {
  if (validate_config(cfg) != KVFOLD_OK) return 0;
  return bytes_required(cfg);
}

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
  if (cfg->device >= n_dev) return KVFOLD_ERR_INVALID_ARG;
  DeviceGuard guard(cfg->device);
  if (guard.err != hipSuccess) return hip_fail(guard.err);

  kvfold_cache* c = new (std::nothrow) kvfold_cache();
  if (!c) return KVFOLD_ERR_OOM;
  c->cfg = *cfg;
  c->elem_bytes = elem_size(cfg->dtype);
  c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  c->kv = nullptr;
  c->owns_kv = false;
  c->kv_bytes = need;
  c->ws_o = nullptr;
  c->ws_ml = nullptr;
  c->ws_rows = 0;
  c->tune_splits = 0;
  c->tune_units_per_wave = 0;
  c->tune_pair_units = 0;
  c->tune_fused_append = 0;
  c->storage_bits = 0;
  c->len.assign((size_t)cfg->n_layers, 0);

  hipDeviceProp_t prop;
  e = hipGetDeviceProperties(&prop, cfg->device);
  if (e != hipSuccess) {
    delete c;
    return hip_fail(e);
  }
  c->n_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

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
    c->ws_rows = ws_rows;
  }
  *out_cache = c;
  return KVFOLD_OK;
}

}  // extern "C"

namespace {

// One fold step; rope_cos / rope_sin both null (inputs used as handed in) or both set.
int step_impl(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new, int32_t n_tokens,
              int64_t pos_offset, const float* rope_cos, const float* rope_sin, void* out, float* lse, void* stream) {
  if (!c || !q || !k_new || !v_new || !out) return KVFOLD_ERR_INVALID_ARG;
  const kvfold_config_t& f = c->cfg;
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
  ap.rope_cos = rope_cos;
  ap.rope_sin = rope_sin;
  ap.elem_is_bf16 = f.dtype == KVFOLD_BF16;

  const Plan pl = make_plan(c, n_tokens, len_prev + n_tokens);
  AttnParams at;
  at.q = q;
  at.k_cache = k_layer;
  at.v_cache = v_layer;
  at.out = out;
  at.lse = lse;
  at.part_o = c->ws_o;
  at.part_ml = c->ws_ml;
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
  at.rope_cos = rope_cos;
  at.rope_sin = rope_sin;
  // The bf16 attention kernel appends by itself when the cache length is a whole number of key tiles (every
  // chunk length that is a multiple of 64) and nothing has to happen to the rows on their way in.
  const bool fused_append = f.dtype == KVFOLD_BF16 && !rope_cos && !c->storage_bits && len_prev % kTileKeys == 0 &&
                            c->tune_fused_append != 1;
  at.k_new = fused_append ? k_new : nullptr;
  at.v_new = fused_append ? v_new : nullptr;
  if (pl.n_splits > 1 && (int64_t)pl.n_splits * n_tokens * f.n_q_heads > c->ws_rows) return KVFOLD_ERR_HIP;  // planner bug guard

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
  if (c->storage_bits) {
    e = launch_storage_roundtrip(ap, c->storage_bits, s);
    if (e != hipSuccess) return hip_fail(e);
  }
  const bool own_append = !fused_append || c->storage_bits;  // something ran between ev[0] and the attention kernel
  if (ev && own_append) (void)hipEventRecord(ev[1], s);
  e = (f.dtype == KVFOLD_BF16) ? launch_attn_bf16(at, f.head_dim, pl.units_per_wave, s) : launch_attn_f32(at, f.head_dim, s);
  if (e != hipSuccess) return hip_fail(e);
  if (ev) (void)hipEventRecord(ev[2], s);
  if (pl.n_splits > 1) {
    CombineParams cp;
    cp.part_o = c->ws_o;
    cp.part_ml = c->ws_ml;
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
  return step_impl(c, layer, q, k_new, v_new, n_tokens, pos_offset, nullptr, nullptr, out, lse, stream);
}

int kvfold_step_rope(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new,
                     int32_t n_tokens, int64_t pos_offset, const float* rope_cos, const float* rope_sin, void* out,
                     float* lse, void* stream) {
  if (!rope_cos || !rope_sin) return KVFOLD_ERR_INVALID_ARG;
  if ((reinterpret_cast<uintptr_t>(rope_cos) | reinterpret_cast<uintptr_t>(rope_sin)) & 15) return KVFOLD_ERR_INVALID_ARG;
  return step_impl(c, layer, q, k_new, v_new, n_tokens, pos_offset, rope_cos, rope_sin, out, lse, stream);
}

int kvfold_step(kvfold_cache_t* c, int layer, const void* q, const void* k_new, const void* v_new, int64_t pos_offset,
                void* out, void* stream) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  return kvfold_step_ex(c, layer, q, k_new, v_new, c->cfg.chunk_tokens, pos_offset, out, nullptr, stream);
}

int kvfold_cache_destroy(kvfold_cache_t* c) {
  if (!c) return KVFOLD_OK;
  int rc = KVFOLD_OK;
  {
    DeviceGuard guard(c->cfg.device);
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
  if (layer < 0 || layer >= c->cfg.n_layers) return KVFOLD_ERR_BAD_LAYER;
  return c->len[(size_t)layer];
}

int kvfold_cache_view(const kvfold_cache_t* c, int layer, void** k_dev, void** v_dev, int64_t* row_stride_elems,
                      int64_t* head_stride_elems) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  const kvfold_config_t& f = c->cfg;
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
  if (layer < -1 || layer >= c->cfg.n_layers) return KVFOLD_ERR_BAD_LAYER;
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
  if (layer < -1 || layer >= c->cfg.n_layers) return KVFOLD_ERR_BAD_LAYER;
  if (new_len < 0) return KVFOLD_ERR_INVALID_ARG;
  if (new_len > c->cfg.capacity_tokens) return KVFOLD_ERR_CAPACITY;
  if (layer == -1)
    for (auto& v : c->len) v = new_len;
  else
    c->len[(size_t)layer] = new_len;
  return KVFOLD_OK;
}

int kvfold_cache_set_storage_roundtrip(kvfold_cache_t* c, int32_t n_bits) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  if (n_bits != 0 && n_bits != 4 && n_bits != 8) return KVFOLD_ERR_INVALID_ARG;
  if (n_bits != 0 && c->cfg.dtype != KVFOLD_BF16) return KVFOLD_ERR_UNSUPPORTED;
  c->storage_bits = n_bits;
  return KVFOLD_OK;
}

int kvfold_cache_set_tuning(kvfold_cache_t* c, int32_t knob, int32_t value) {
  if (!c) return KVFOLD_ERR_INVALID_ARG;
  switch (knob) {
    case KVFOLD_TUNE_SPLITS:
      if (value < 0 || value > kMaxSplits) return KVFOLD_ERR_INVALID_ARG;
      c->tune_splits = value;
      return KVFOLD_OK;
    case KVFOLD_TUNE_PAIR_UNITS:
      if (value < 0 || value > 2) return KVFOLD_ERR_INVALID_ARG;
      c->tune_pair_units = value;
      return KVFOLD_OK;
    case KVFOLD_TUNE_FUSED_APPEND:
      if (value < 0 || value > 1) return KVFOLD_ERR_INVALID_ARG;
      c->tune_fused_append = value;
      return KVFOLD_OK;
    case KVFOLD_TUNE_UNITS_PER_WAVE:
      if (value < 0 || value > 2) return KVFOLD_ERR_INVALID_ARG;
      c->tune_units_per_wave = value;
      return KVFOLD_OK;
    default:
      return KVFOLD_ERR_INVALID_ARG;
  }
}

int kvfold_cache_plan(const kvfold_cache_t* c, int32_t n_tokens, int64_t len_after, int32_t* n_workgroups,
                      int32_t* n_splits) {
  if (!c || n_tokens < 1 || n_tokens > c->cfg.chunk_tokens || len_after < n_tokens ||
      len_after > c->cfg.capacity_tokens)
    return KVFOLD_ERR_INVALID_ARG;
  const Plan pl = make_plan(c, n_tokens, len_after);
  if (n_workgroups) *n_workgroups = pl.n_wgs;
  if (n_splits) *n_splits = pl.n_splits;
  return KVFOLD_OK;
}

int kvfold_cache_profile_begin(kvfold_cache_t* c, int32_t max_steps) {
  if (!c || max_steps < 1 || max_steps > (1 << 20) || c->prof_max_steps > 0) return KVFOLD_ERR_INVALID_ARG;
  DeviceGuard guard(c->cfg.device);
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
  DeviceGuard guard(c->cfg.device);
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

int kvfold_plan_for(const kvfold_config_t* cfg, int32_t n_compute_units, int32_t n_tokens, int64_t len_after,
                    int32_t* n_workgroups, int32_t* n_splits, int32_t* units_per_wave) {
  const int rc = validate_config(cfg);
  if (rc != KVFOLD_OK) return rc;
  if (n_compute_units < 1 || n_tokens < 1 || n_tokens > cfg->chunk_tokens || len_after < n_tokens ||
      len_after > cfg->capacity_tokens)
    return KVFOLD_ERR_INVALID_ARG;
  kvfold_cache c{};  // host fields only: nothing here touches a device
  c.cfg = *cfg;
  c.elem_bytes = elem_size(cfg->dtype);
  c.ws_rows = workspace_rows(cfg);
  c.n_cu = n_compute_units;
  const Plan pl = make_plan(&c, n_tokens, len_after);
  if (n_workgroups) *n_workgroups = pl.n_wgs;
  if (n_splits) *n_splits = pl.n_splits;
  if (units_per_wave) *units_per_wave = pl.units_per_wave;
  return KVFOLD_OK;
}

const char* kvfold_status_string(int status) {
  switch (status) {
    case KVFOLD_OK: return "ok";
    case KVFOLD_ERR_INVALID_ARG: return "invalid argument";
    case KVFOLD_ERR_BAD_LAYER: return "layer out of range";
    case KVFOLD_ERR_POSITION: return "pos_offset does not continue the cache";
    case KVFOLD_ERR_CAPACITY: return "cache capacity exceeded";
    case KVFOLD_ERR_UNSUPPORTED: return "unsupported configuration";
    case KVFOLD_ERR_OOM: return "out of device memory or buffer too small";
    case KVFOLD_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int kvfold_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
