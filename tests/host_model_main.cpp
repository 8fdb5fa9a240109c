// Host-only test program (no GPU, no HIP): built from the library's HIP-free sources and the C oracle with
// -fsanitize=address,undefined by tests/test_host_model.py.
//
//  1. A host model of the attention kernels' key-range walk.  The kernels' tile arithmetic lives in
//     kvfold_consts.h (workgroup_rows, tile_map, key_range, dma_row) and the launch geometry in the planner;
//     both are used here exactly as the kernels use them.  For many shapes -- chunk length, cache length, group
//     size, prefix splits, units per wavefront, fused append or not, plain and sink + sliding-window steps --
//     every workgroup's pieces are walked, ring run-ahead included, and checked:
//       * every DMA source row lies inside what exists (cache rows below len_prev when the chunk's rows are not
//         in the cache yet, else below len_prev + C; chunk rows below C), with 32-bit offsets that do not wrap;
//       * a row that a query of the workgroup can see is fetched unclamped, from the right place;
//       * the pieces of all splits together cover every visible key of every row of the workgroup exactly once.
//  2. The planner and validate_config over a sweep of configurations (sanitizers watch the arithmetic).
//  3. The oracle on tiny inputs, plain and windowed (sanitizers watch its indexing).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../paper_2605_12471_amd/csrc/kvfold_plan.h"

extern "C" {
int kvfold_oracle_attend_rows(const double*, const double*, int64_t, int64_t, int64_t, const double*, int64_t, int64_t,
                              int64_t, double, const int64_t*, int64_t, double*, double*, double*);
int kvfold_oracle_attend_rows_window(const double*, const double*, int64_t, int64_t, int64_t, const double*, int64_t,
                                     int64_t, int64_t, double, int64_t, int64_t, const int64_t*, int64_t, double*,
                                     double*, double*);
int kvfold_oracle_append_bytes(unsigned char*, int64_t, int64_t, int64_t, int64_t, const unsigned char*, int64_t, int64_t);
}

using namespace kvfold;

static long g_checks = 0;
#define REQUIRE(cond, ...)                                   \
  do {                                                       \
    ++g_checks;                                              \
    if (!(cond)) {                                           \
      std::fprintf(stderr, "FAILED %s:%d: %s\n  ", __FILE__, __LINE__, #cond); \
      std::fprintf(stderr, __VA_ARGS__);                     \
      std::fprintf(stderr, "\n");                            \
      std::exit(1);                                          \
    }                                                        \
  } while (0)

// Ring depth of the bf16 kernels: the refill runs NV + 1 tiles ahead of the tile being read.
static const int kRunAhead = 4;

static void walk_step(const kvfold_config_t& cfg, int n_cu, int n_tokens, int64_t len_prev, int n_sink, int64_t window,
                      int force_splits, int force_upw) {
  PlanCtx pc{};
  pc.cfg = cfg;
  pc.ws_rows = workspace_rows(&cfg);
  pc.n_cu = n_cu;
  pc.tune_splits = force_splits;
  pc.tune_units_per_wave = force_upw;
  const int64_t len_after = len_prev + n_tokens;
  const Plan pl = make_plan(pc, n_tokens, len_after, n_sink, window);
  const bool fused = fused_append_applies(pc, n_tokens, len_prev, false);
  const int G = cfg.n_q_heads / cfg.n_kv_heads;
  const int upw_wg = kUnitsPerWg * pl.units_per_wave;
  const int row_bytes = cfg.head_dim * elem_size(cfg.dtype);
  REQUIRE(pl.n_splits >= 1 && pl.n_splits <= kMaxSplits && pl.tiles_per_split >= 1, "plan");
  REQUIRE(pl.n_splits == 1 || (int64_t)pl.n_splits * n_tokens * cfg.n_q_heads <= pc.ws_rows, "workspace");
  REQUIRE(pl.n_wgs == cfg.n_kv_heads * pl.wgs_per_head * pl.n_splits, "grid");
  if (window > 0) REQUIRE(!pl.pair_units && !pl.pair_order, "pairing under a window");

  std::vector<int> seen((size_t)len_after);
  for (int ug = 0; ug < pl.wgs_per_head; ++ug) {
    RowRange rr;
    if (pl.pair_units) {  // an early and a late unit per wavefront: the workgroup's keys run up to the late unit's rows
      rr.row_lo = 0;
      int ulast = pl.units_per_head - 1 - ug * kUnitsPerWg;
      if (ulast < 0) ulast = 0;
      rr.row_hi = (ulast / G) * kRowsPerUnit + kRowsPerUnit - 1;
      if (rr.row_hi > n_tokens - 1) rr.row_hi = n_tokens - 1;
    } else {
      rr = workgroup_rows(ug, upw_wg, pl.units_per_head, G, n_tokens);
    }
    const TileMap tm = tile_map(len_prev, rr.row_lo, rr.row_hi, n_sink, window);
    REQUIRE(tm.ntiles >= 1 && tm.skip >= 0 && tm.ns_t >= 0, "tile map");
    REQUIRE((int64_t)pl.n_splits * pl.tiles_per_split >= tm.ntiles, "pieces do not cover the workgroup's %d tiles (%d x %d)",
            tm.ntiles, pl.n_splits, pl.tiles_per_split);
    std::fill(seen.begin(), seen.end(), 0);
    for (int split = 0; split < pl.n_splits; ++split) {
      const KeyRange kr = key_range(tm, split, pl.tiles_per_split, len_prev, n_tokens, fused);
      if (kr.t_begin >= kr.t_end) continue;  // an empty piece touches nothing
      // (a piece that never reads the chunk as handed in ends below len_prev, so the clamp keeps it there too)
      const int64_t readable_cache = fused ? len_prev : len_after;
      REQUIRE((int64_t)kr.row_lim < len_after, "row_lim");
      for (int t = kr.t_begin; t < kr.t_end + kRunAhead; ++t) {
        const int tp = t + (t >= tm.ns_t ? tm.skip : 0);
        for (int row = 0; row < kTileKeys; ++row) {
          const DmaRow d = dma_row(kr, tp, row);
          const int64_t key = (int64_t)tp * kTileKeys + row;  // the key this ring row stands for
          if (d.from_chunk) {
            REQUIRE(fused && (int64_t)d.row < n_tokens, "chunk row %u out of %d", d.row, n_tokens);
            REQUIRE((uint64_t)d.row * cfg.n_kv_heads * row_bytes + row_bytes <= (1ull << 32), "32-bit chunk offset wraps");
          } else {
            REQUIRE((int64_t)d.row < readable_cache, "cache row %u not readable (%lld rows are)", d.row, (long long)readable_cache);
            REQUIRE((uint64_t)d.row * row_bytes + row_bytes <= (1ull << 32), "32-bit cache offset wraps");
          }
          if (t < kr.t_end && key < len_after && key <= len_prev + rr.row_hi) {
            // inside the piece and not beyond the workgroup's last row: must be the key itself
            const int64_t got = d.from_chunk ? len_prev + d.row : d.row;
            REQUIRE(got == key, "tile %d (physical %d) row %d reads key %lld instead of %lld", t, tp, row, (long long)got,
                    (long long)key);
            REQUIRE(d.from_chunk == (fused && key >= len_prev), "wrong source for key %lld", (long long)key);
            seen[(size_t)key]++;
          }
        }
      }
    }
    // every key some row of the workgroup can see was fetched exactly once
    for (int r = rr.row_lo; r <= rr.row_hi; ++r) {
      const int64_t p = len_prev + r;
      for (int64_t j = 0; j <= p; ++j) {
        const bool vis = window <= 0 || j < n_sink || j > p - window;
        if (vis) REQUIRE(seen[(size_t)j] == 1, "key %lld visible to row %d fetched %d times (ug %d)", (long long)j, r, seen[(size_t)j], ug);
      }
    }
    for (int64_t j = 0; j < len_after; ++j) REQUIRE(seen[(size_t)j] <= 1, "key %lld fetched twice", (long long)j);
  }
}

static kvfold_config_t make_cfg(int Hq, int Hkv, int d, int C, int64_t cap, int dtype) {
  kvfold_config_t c{};
  c.struct_size = sizeof(c);
  c.n_layers = 1;
  c.n_q_heads = Hq;
  c.n_kv_heads = Hkv;
  c.head_dim = d;
  c.chunk_tokens = C;
  c.capacity_tokens = cap;
  c.dtype = dtype;
  return c;
}

static void model_sweep() {
  const int heads[][2] = {{4, 1}, {7, 1}, {6, 3}, {32, 8}, {2, 2}};
  const int chunks[] = {1, 16, 33, 64, 100, 256, 1000};
  const int64_t prefixes[] = {0, 63, 64, 500, 1024, 5000};
  const int64_t windows[][2] = {{0, 0}, {4, 1020}, {0, 1}, {4, 1}, {1, 33}, {70, 50}, {130, 129}, {0, 1 << 20}};
  long steps = 0;
  for (auto& h : heads)
    for (int C : chunks)
      for (int64_t Lp : prefixes)
        for (auto& w : windows)
          for (int dtype : {(int)KVFOLD_BF16, (int)KVFOLD_F32}) {
            kvfold_config_t cfg = make_cfg(h[0], h[1], 128, C, Lp + C, dtype);
            REQUIRE(validate_config(&cfg) == KVFOLD_OK, "config");
            for (int splits : {0, 2, 5})
              for (int upw : {0, 1, 2}) {
                if (dtype == KVFOLD_F32 && upw == 2) continue;
                if (splits > 0 && (int64_t)splits * C * h[0] > workspace_rows(&cfg)) continue;
                walk_step(cfg, 256, C, Lp, (int)w[0], w[1], splits, upw);
                ++steps;
              }
          }
  // the benchmark's shapes at their real sizes, plain and with the streaming baseline's window
  struct { int Hq, Hkv, C; int64_t Lp; } big[] = {{32, 8, 2048, 14336}, {32, 8, 256, 130816}, {32, 8, 4096, 126976},
                                                 {28, 4, 128, 65408}, {28, 4, 8192, 57344}, {32, 8, 16, 131056}, {32, 8, 1, 131071}};
  for (auto& b : big)
    for (auto& w : {std::pair<int, int64_t>{0, 0}, {4, 1020}}) {
      kvfold_config_t cfg = make_cfg(b.Hq, b.Hkv, 128, b.C, b.Lp + b.C, KVFOLD_BF16);
      walk_step(cfg, 256, b.C, b.Lp, w.first, w.second, 0, 0);
      ++steps;
    }
  std::printf("host model: %ld steps walked\n", steps);
}

static void planner_sweep() {
  long n = 0;
  for (int Hkv : {1, 2, 4, 8, 64, 32767})
    for (int G : {1, 4, 7})
      for (int d : {64, 128})
        for (int64_t cap : {(int64_t)1, (int64_t)4096, (int64_t)131072, (int64_t)1 << 24, (int64_t)1 << 30})
          for (int C : {1, 64, 4096, 1 << 20})
            for (int dtype : {(int)KVFOLD_F32, (int)KVFOLD_BF16, 7}) {
              kvfold_config_t cfg = make_cfg(Hkv * G, Hkv, d, C, cap, dtype);
              const int rc = validate_config(&cfg);
              if (rc != KVFOLD_OK) {
                REQUIRE(kvfold_cache_bytes_required(&cfg) == 0, "bytes of an invalid config");
                continue;
              }
              REQUIRE(kvfold_cache_bytes_required(&cfg) == (size_t)2 * Hkv * cap * d * elem_size(dtype), "bytes");
              for (int64_t len_after : {(int64_t)C, cap})
                for (auto& w : {std::pair<int, int64_t>{0, 0}, {4, 1020}, {1 << 20, (int64_t)1 << 30}}) {
                  if (len_after < C || len_after > cap) continue;
                  kvfold_plan_t out;
                  const int prc = kvfold_plan_for(&cfg, 256, C, len_after, w.first, w.second, &out);
                  REQUIRE(prc == KVFOLD_OK, "plan_for rc %d", prc);
                  REQUIRE(out.n_workgroups >= 1 && out.n_splits >= 1 && out.tiles_per_split >= 1, "plan_for values");
                  REQUIRE((int64_t)out.n_splits * out.tiles_per_split * kTileKeys >= (w.second ? 1 : len_after), "plan_for tiles");
                  ++n;
                }
            }
  std::printf("planner: %ld plans\n", n);
}

static void oracle_tiny() {
  const int64_t Hq = 4, Hkv = 2, d = 8, cap = 40, C = 9, len_prev = 31;
  std::vector<double> K((size_t)Hkv * cap * d), V(K.size()), q((size_t)C * Hq * d);
  unsigned s = 12345;
  auto rnd = [&]() { s = s * 1664525u + 1013904223u; return (double)(s >> 8) / (1 << 24) - 0.5; };
  for (auto& x : K) x = rnd();
  for (auto& x : V) x = rnd();
  for (auto& x : q) x = rnd();
  std::vector<int64_t> rows = {0, 3, 8};
  std::vector<double> out(rows.size() * Hq * d), lse(rows.size() * Hq), w(rows.size() * Hq * (len_prev + C));
  REQUIRE(kvfold_oracle_attend_rows(K.data(), V.data(), Hkv, cap, d, q.data(), C, Hq, len_prev, 0.35, rows.data(),
                                    (int64_t)rows.size(), out.data(), lse.data(), w.data()) == 0, "oracle plain");
  std::vector<double> out2(out.size()), lse2(lse.size()), w2(w.size());
  REQUIRE(kvfold_oracle_attend_rows_window(K.data(), V.data(), Hkv, cap, d, q.data(), C, Hq, len_prev, 0.35, 0, 1000,
                                           rows.data(), (int64_t)rows.size(), out2.data(), lse2.data(), w2.data()) == 0, "oracle window");
  REQUIRE(std::memcmp(out.data(), out2.data(), out.size() * sizeof(double)) == 0, "an all-covering window is the plain step");
  REQUIRE(kvfold_oracle_attend_rows_window(K.data(), V.data(), Hkv, cap, d, q.data(), C, Hq, len_prev, 0.35, 2, 5,
                                           rows.data(), (int64_t)rows.size(), out2.data(), lse2.data(), w2.data()) == 0, "oracle window");
  for (size_t r = 0; r < rows.size(); ++r)
    for (int64_t h = 0; h < Hq; ++h) {
      int nz = 0;
      for (int64_t j = 0; j < len_prev + C; ++j) nz += w2[(r * Hq + h) * (len_prev + C) + j] > 0;
      REQUIRE(nz == 7, "2 sinks + 5 recent keys carry weight, got %d", nz);
    }
  REQUIRE(kvfold_oracle_attend_rows(K.data(), V.data(), Hkv, cap, d, q.data(), C, Hq, 32, 0.35, rows.data(), 3, out.data(),
                                    lse.data(), nullptr) == -1, "beyond capacity");
  // append: bytes land head-major at rows [len, len + C)
  std::vector<unsigned char> cache((size_t)Hkv * cap * d * 2, 0), chunk((size_t)C * Hkv * d * 2);
  for (size_t i = 0; i < chunk.size(); ++i) chunk[i] = (unsigned char)(i * 7 + 1);
  REQUIRE(kvfold_oracle_append_bytes(cache.data(), Hkv, cap, d, len_prev, chunk.data(), C, 2) == 0, "append");
  REQUIRE(cache[((size_t)1 * cap + len_prev + 2) * d * 2 + 3] == chunk[((size_t)2 * Hkv + 1) * d * 2 + 3], "append layout");
  REQUIRE(kvfold_oracle_append_bytes(cache.data(), Hkv, cap, d, len_prev, chunk.data(), C + 1, 2) == -1, "append beyond capacity");
  std::printf("oracle: tiny cases ok\n");
}

int main() {
  model_sweep();
  planner_sweep();
  oracle_tiny();
  std::printf("ok: %ld checks\n", g_checks);
  return 0;
}
