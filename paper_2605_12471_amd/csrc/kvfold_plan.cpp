// Configuration checks, byte accounting and the launch planner of libkvfold: everything the host decides
// before a kernel is launched.  No HIP in this file.
#include "kvfold_plan.h"

#include <algorithm>
#include <cmath>

namespace kvfold {

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
  // the append kernels put (KV head, K or V) on the grid's second dimension (at most 65535 blocks)
  if (c->n_kv_heads > 32767) return KVFOLD_ERR_UNSUPPORTED;
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

// split workspace: room for kMaxSplits pieces of one chunk, capped
int64_t workspace_rows(const kvfold_config_t* cfg) {
  const int64_t rows = (int64_t)cfg->chunk_tokens * cfg->n_q_heads;
  int64_t ws_rows = rows * kMaxSplits;
  if (ws_rows > kMaxSplitRows) ws_rows = kMaxSplitRows;
  if (ws_rows < 2 * rows) ws_rows = 0;  // chunks this large never need a split
  return ws_rows;
}

// The fused append reads the chunk's rows, [C][Hkv][d], with 32-bit byte offsets from the KV head's first row:
// the largest is below C * Hkv * row_bytes, which therefore has to stay below 2^32.
bool fused_append_applies(const PlanCtx& c, int n_tokens, int64_t len_prev, bool rope) {
  const kvfold_config_t& f = c.cfg;
  if (f.dtype != KVFOLD_BF16 || rope || c.storage_bits || c.tune_fused_append == 1) return false;
  (void)len_prev;  // any cache length: a tile that straddles the cache's end is filled from both sides
  const int64_t chunk_bytes = (int64_t)n_tokens * f.n_kv_heads * f.head_dim * elem_size(f.dtype);
  return chunk_bytes < ((int64_t)1 << 32);
}

namespace {

// Launch geometry for `upw` units per wavefront: enough prefix splits to put at least `target`
// workgroups on the chip when the unsplit grid has fewer (a forced split count overrides that).
Plan plan_with(const PlanCtx& c, int n_tokens, int64_t len_after, int upw, int n_sink, int64_t window) {
  const kvfold_config_t& f = c.cfg;
  const int G = f.n_q_heads / f.n_kv_heads;
  Plan pl;
  pl.pair_order = 0;
  pl.pair_units = 0;
  pl.units_per_head = G * ((n_tokens + kRowsPerUnit - 1) / kRowsPerUnit);
  pl.units_per_wave = upw;
  const int per_wg = kUnitsPerWg * upw;
  pl.wgs_per_head = (pl.units_per_head + per_wg - 1) / per_wg;
  const int64_t base = (int64_t)f.n_kv_heads * pl.wgs_per_head;
  // tiles of the longest key range of any workgroup (the kernels cut exactly this many into pieces), and the
  // (row, key) pairs of the step
  int ntiles = (int)((len_after + kTileKeys - 1) / kTileKeys);
  double pairs = (double)n_tokens * ((double)len_after - 0.5 * n_tokens);
  if (window > 0) {
    ntiles = 1;
    for (int ug = 0; ug < pl.wgs_per_head; ++ug) {
      const RowRange rr = workgroup_rows(ug, per_wg, pl.units_per_head, G, n_tokens);
      ntiles = std::max(ntiles, tile_map(len_after - n_tokens, rr.row_lo, rr.row_hi, n_sink, window).ntiles);
    }
    const double per_row = std::min((double)len_after - 0.5 * n_tokens, (double)n_sink + (double)window);
    pairs = (double)n_tokens * per_row;
  }
  int64_t s_max = c.tune_splits > 0 ? ntiles : ntiles / kMinTilesPerSplit;  // a forced count only needs a tile each
  const int64_t rows = (int64_t)n_tokens * f.n_q_heads;
  if (c.ws_rows / rows < s_max) s_max = c.ws_rows / rows;
  if (s_max > kMaxSplits) s_max = kMaxSplits;
  if (s_max < 1) s_max = 1;
  int64_t s = 1;
  pl.est_seconds = 0.0;
  if (c.tune_splits > 0) {
    s = c.tune_splits;
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
    //  * Matrix work counts the padding of the last workgroup of a KV head (units that do not exist are computed
    //    all the same), and 10 % more in the one-unit kernel, where every LDS fragment feeds one MFMA instead of two.
    //    A one-unit grid of at most one workgroup per CU runs one wavefront per SIMD with nothing to overlap with:
    //    7 % less than two per CU deliver between them (measured on the C = 128, G = 7 fold: 8 pieces on 224 CUs
    //    beat 18 pieces on all 256 twice over by 3 %).
    const double pad = (double)((int64_t)pl.wgs_per_head * per_wg) / (double)pl.units_per_head;
    const double kernel_cost = upw == 2 ? 1.0 : 1.1;
    const double flops = 4.0 * f.n_q_heads * f.head_dim * pairs * pad * kernel_cost;
    const double kv_rows = window > 0 ? std::min((double)len_after, (double)ntiles * kTileKeys * pl.wgs_per_head) : (double)len_after;
    const double kv_bytes = 2.0 * f.n_kv_heads * f.head_dim * (double)elem_size(f.dtype) * kv_rows;
    const double t_attn = std::max(flops / (f.dtype == KVFOLD_BF16 ? 1.35e15 : 1.2e14), kv_bytes / 5e12);  // bf16 / fp32 MFMA rates
    double best = 1e30;
    for (int64_t cand = 1; cand <= s_max; ++cand) {
      // only split counts that whole tiles can realise; the last piece may be shorter than the others, and the
      // launch lasts as long as the longest
      const int64_t tps = (ntiles + cand - 1) / cand;
      if ((ntiles + tps - 1) / tps != cand) continue;
      const double uneven = (double)(tps * cand) / (double)ntiles;
      const int64_t w = base * cand;
      const bool one_per_cu = upw == 1 && w <= (int64_t)c.n_cu;
      const int64_t slots = (int64_t)c.n_cu * (upw == 1 && !one_per_cu ? 2 : 1);
      const int64_t rounds = (w + slots - 1) / slots;
      double fill = (double)w / (double)(rounds * slots);
      if (cand == 1 && rounds >= 2 && window <= 0) {
        const double w_min = (double)(len_after - n_tokens) + kRowsPerUnit, w_mean = (double)len_after - 0.5 * n_tokens;
        fill = (double)w * w_mean / ((double)w * w_mean + (double)(rounds * slots - w) * w_min);
      }
      const double rate = std::min(1.41 * fill, std::pow(fill, 0.3)) * (one_per_cu ? 0.93 : 1.0);
      const double merge = cand > 1 ? (double)cand * rows * (f.head_dim + 2) * 8.0 / 4e12 + 6e-6 : 0.0;
      const double t = t_attn * uneven / rate * (1.0 + 0.03 / (double)rounds) + 8e-6 * (double)rounds + merge;
      if (t < best * 0.995) {
        best = t;
        s = cand;
      }
    }
    pl.est_seconds = best;
  }
  if (s > s_max) s = s_max;
  pl.tiles_per_split = (int)((ntiles + s - 1) / s);
  if (pl.tiles_per_split < 1) pl.tiles_per_split = 1;
  pl.n_splits = (ntiles + pl.tiles_per_split - 1) / pl.tiles_per_split;
  if (pl.n_splits < 1) pl.n_splits = 1;
  pl.n_wgs = (int)(base * pl.n_splits);
  return pl;
}

Plan choose_plan(const PlanCtx& c, int n_tokens, int64_t len_after, int n_sink, int64_t window) {
  const kvfold_config_t& f = c.cfg;
  if (f.dtype != KVFOLD_BF16) return plan_with(c, n_tokens, len_after, 1, n_sink, window);
  if (c.tune_units_per_wave) return plan_with(c, n_tokens, len_after, c.tune_units_per_wave, n_sink, window);
  Plan p1 = plan_with(c, n_tokens, len_after, 1, n_sink, window);
  // Prefix shorter than the chunk: the causal part makes late token blocks several times as long as early
  // ones.  If the one-unit-per-wavefront grid is resident at once (two workgroups per CU), pair heavy with
  // light workgroups on a CU (measured faster than pairing units inside the two-unit kernel only here).
  const int64_t wgs1 = (int64_t)f.n_kv_heads * p1.wgs_per_head;
  if (c.tune_splits == 0 && window <= 0 && len_after < 2 * (int64_t)n_tokens && wgs1 <= 2 * (int64_t)c.n_cu &&
      wgs1 > (int64_t)c.n_cu && p1.n_splits == 1) {
    p1.pair_order = 1;
    return p1;
  }
  // Two units per wavefront is the faster kernel (every LDS fragment feeds two MFMAs) whenever it
  // can fill the chip, if need be by splitting the prefix; one unit per wavefront is for grids too
  // small for that, and for chunks so short that half of the two-unit workgroup would idle.
  const Plan p2 = plan_with(c, n_tokens, len_after, 2, n_sink, window);
  const int64_t padded1 = (int64_t)p1.wgs_per_head * kUnitsPerWg, padded2 = (int64_t)p2.wgs_per_head * kUnitsPerWg * 2;
  if (padded2 * 5 > padded1 * 6) return p1;                                   // more than 20 % extra padding
  if ((int64_t)p2.n_wgs * 4 < (int64_t)c.n_cu * 3 && p1.n_wgs > p2.n_wgs) return p1;  // cannot fill the chip
  // Some extra padding (odd group sizes: 28 units of a G = 7 head at C = 128 fill 3.5 two-unit workgroups): the
  // time estimates of the two grids decide.
  if (padded2 > padded1 && c.tune_splits == 0 && p1.est_seconds < p2.est_seconds) return p1;
  return p2;
}

}  // namespace

Plan make_plan(const PlanCtx& c, int n_tokens, int64_t len_after, int n_sink, int64_t window) {
  Plan pl = choose_plan(c, n_tokens, len_after, n_sink, window);
  // Two-unit kernel, a single round of workgroups: the causal part makes the last token block's wavefronts
  // longer than the first's (100 % on an empty cache, 6 % after 8 chunks) and nothing evens that out; pair
  // an early and a late row block in every wavefront instead (the late one finishes alone, at the
  // efficiency of a one-unit step).  Measured: +7 % down to +0.5 % at 31 chunks of prefix, even at 63; with
  // a split prefix (only the last pieces hold the causal part) +0.5 to 2 %, never a loss.  With several
  // rounds the dispatcher balances heaviest-first workgroups by itself and pairing only costs.  Under a
  // sliding window every row block has the same number of keys and there is nothing to pair.
  if (c.cfg.dtype == KVFOLD_BF16 && pl.units_per_wave == 2 && c.tune_pair_units != 1 && window <= 0) {
    if (c.tune_pair_units == 2 || pl.n_wgs <= c.n_cu) pl.pair_units = 1;
  }
  return pl;
}

}  // namespace kvfold

using namespace kvfold;

extern "C" {

size_t kvfold_cache_bytes_required(const kvfold_config_t* cfg) {
  if (validate_config(cfg) != KVFOLD_OK) return 0;
  return bytes_required(cfg);
}

int kvfold_plan_for(const kvfold_config_t* cfg, int32_t n_compute_units, int32_t n_tokens, int64_t len_after,
                    int32_t n_sink, int64_t window, kvfold_plan_t* out) {
  const int rc = validate_config(cfg);
  if (rc != KVFOLD_OK) return rc;
  if (n_compute_units < 1 || n_tokens < 1 || n_tokens > cfg->chunk_tokens || len_after < n_tokens ||
      len_after > cfg->capacity_tokens || n_sink < 0 || window < 0 || !out)
    return KVFOLD_ERR_INVALID_ARG;
  PlanCtx c{};
  c.cfg = *cfg;
  c.ws_rows = workspace_rows(cfg);
  c.n_cu = n_compute_units;
  const Plan pl = make_plan(c, n_tokens, len_after, n_sink, window);
  out->n_workgroups = pl.n_wgs;
  out->n_splits = pl.n_splits;
  out->units_per_wave = pl.units_per_wave;
  out->tiles_per_split = pl.tiles_per_split;
  out->fused_append = fused_append_applies(c, n_tokens, len_after - n_tokens, false) ? 1 : 0;
  out->pair_units = pl.pair_units;
  out->pair_order = pl.pair_order;
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
    case KVFOLD_ERR_SCRATCH: return "step does not fit the static scratch buffer";
    default: return "unknown status";
  }
}

}  // extern "C"
