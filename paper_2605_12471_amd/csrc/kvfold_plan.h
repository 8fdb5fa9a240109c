// Host-only part of libkvfold that needs no HIP: configuration checks, byte accounting and the launch
// planner.  Built into the library and, as plain C++ with the host sanitizers, into a test program.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/kvfold.h"
#include "kvfold_consts.h"

namespace kvfold {

constexpr int64_t kMaxSplitRows = 1 << 19;  // cap on S * C * Hq rows held in a cache's split workspace
constexpr int kMaxSplits = 64;
constexpr int kMinTilesPerSplit = 8;

// What the planner needs to know of a cache (all host values).
struct PlanCtx {
  kvfold_config_t cfg;
  int64_t ws_rows;  // (row, split) pairs the split workspace in use can hold
  int n_cu;
  int tune_splits, tune_units_per_wave, tune_pair_units, tune_fused_append;
  int storage_bits;
};

struct Plan {
  int units_per_wave, units_per_head, wgs_per_head, n_splits, tiles_per_split, n_wgs, pair_order, pair_units;
  double est_seconds;  // the planner's time estimate of the step (0 when the split count was forced)
};

int elem_size(int dtype);
int validate_config(const kvfold_config_t* c);
size_t bytes_required(const kvfold_config_t* c);
// (row, split) pairs of the workspace that kvfold_cache_create reserves
int64_t workspace_rows(const kvfold_config_t* cfg);
// Launch geometry of one step of n_tokens rows that leaves the cache at len_after rows; window > 0 selects the
// sink + sliding-window step (n_sink first keys plus the last `window` keys of every row).
Plan make_plan(const PlanCtx& c, int n_tokens, int64_t len_after, int n_sink, int64_t window);
// Whether the bf16 attention kernel does the append itself for this step.
bool fused_append_applies(const PlanCtx& c, int n_tokens, int64_t len_prev, bool rope);

}  // namespace kvfold
