// Tile geometry shared by the kernels and the host-side planner (no HIP types here: the planner is built
// as plain C++ as well, for host-only tests).
#pragma once

namespace kvfold {

// Rows of one (query head, 32-token block) pair are the unit of work of one wavefront.
constexpr int kRowsPerUnit = 32;
// Wavefronts (units) per workgroup of the attention kernels.
constexpr int kUnitsPerWg = 4;
// Keys per K/V tile staged through LDS.
constexpr int kTileKeys = 64;
// The hardware hands workgroup b to XCD b % 8.
constexpr int kNumXcd = 8;


#if defined(__HIP__)
#define KVFOLD_HD __host__ __device__ inline __attribute__((always_inline))
#else
#define KVFOLD_HD inline
#endif

// Chunk rows [row_lo, row_hi] owned by workgroup `ug` of a KV head: its `upw_wg` consecutive units, ordered
// token-block-major, head-minor (unit u = token block u / G, head u % G of the group of G query heads).
struct RowRange {
  int row_lo, row_hi;
};
KVFOLD_HD RowRange workgroup_rows(int ug, int upw_wg, int units_per_head, int G, int n_tokens) {
  int ufirst = ug * upw_wg, ulast = ufirst + upw_wg - 1;
  if (ulast > units_per_head - 1) ulast = units_per_head - 1;
  if (ufirst > ulast) ufirst = ulast;
  if (ufirst < 0) ufirst = 0;
  if (ulast < 0) ulast = 0;
  RowRange r;
  r.row_lo = (ufirst / G) * kRowsPerUnit;
  r.row_hi = (ulast / G) * kRowsPerUnit + kRowsPerUnit - 1;
  if (r.row_hi > n_tokens - 1) r.row_hi = n_tokens - 1;
  if (r.row_lo > r.row_hi) r.row_lo = r.row_hi;
  return r;
}

// Key tiles a workgroup walks.  Plain step (window <= 0): physical tiles [0, ntiles) cover keys
// [0, len_prev + row_hi].  Sink + sliding-window step: the row at absolute position p sees keys j < n_sink and
// p - window < j <= p, so the workgroup needs the sink tiles [0, ns_t) and the tiles from the one that holds key
// len_prev + row_lo - window + 1 on; the `skip` tiles in between are never touched.  The kernels count LOGICAL
// tiles 0 .. ntiles-1; logical tile t is physical tile t + (t >= ns_t ? skip : 0).
struct TileMap {
  int ns_t, skip, ntiles;
};
KVFOLD_HD TileMap tile_map(long long len_prev, int row_lo, int row_hi, int n_sink, long long window) {
  const int nt_phys = (int)((len_prev + row_hi + 1 + kTileKeys - 1) / kTileKeys);
  TileMap tm;
  tm.ns_t = 0;
  tm.skip = 0;
  tm.ntiles = nt_phys;
  if (window <= 0) return tm;
  long long lb = len_prev + row_lo - window + 1;
  if (lb < 0) lb = 0;
  int ns_t = (n_sink + kTileKeys - 1) / kTileKeys;
  if (ns_t > nt_phys) ns_t = nt_phys;
  int tw0 = (int)(lb / kTileKeys);
  if (tw0 < ns_t) tw0 = ns_t;
  tm.ns_t = ns_t;
  tm.skip = tw0 - ns_t;
  tm.ntiles = nt_phys - tm.skip;
  return tm;
}


// Piece `split` of a workgroup's logical tiles, [t_begin, t_end), and what the DMA of its K/V tiles may touch.
// The LDS ring runs a few tiles ahead and knows no end, so every source row is clamped to row_lim, the last row
// of the piece that exists (the cache holds rows [0, len_prev + n_tokens)).  With the append fused into the
// attention kernel the chunk's rows are not in the cache yet: rows from chunk_row0 = len_prev on are read from the
// rows as handed in, [n_tokens][Hkv][d], counted from the chunk's first row -- unless the piece ends before the
// chunk begins, in which case nothing is ever read from there.  Physical tiles from t_new on lie wholly in the
// chunk; when len_prev is not a multiple of the tile, tile t_straddle = t_new - 1 holds rows of both.
struct KeyRange {
  int t_begin, t_end;   // logical tiles
  unsigned row_lim;     // last row (cache numbering) a DMA of this piece may read
  unsigned chunk_row0;  // first row that comes from the chunk as handed in (0xffffffff: none does)
  int t_new;            // first physical tile that lies wholly in the chunk (INT_MAX: none)
  int t_straddle;       // physical tile with rows on both sides of chunk_row0 (-1: none)
};
KVFOLD_HD KeyRange key_range(const TileMap& tm, int split, int tiles_per_split, long long len_prev, int n_tokens, bool fused) {
  KeyRange k;
  k.t_begin = split * tiles_per_split;
  k.t_end = k.t_begin + tiles_per_split;
  if (k.t_end > tm.ntiles) k.t_end = tm.ntiles;
  const int last = k.t_end - 1;  // (only used when the piece is not empty)
  const long long row_end = (long long)(last + (last >= tm.ns_t ? tm.skip : 0)) * kTileKeys + kTileKeys - 1;
  const long long Lm1 = len_prev + n_tokens - 1;
  const long long lim = row_end < Lm1 ? row_end : Lm1;
  k.row_lim = (unsigned)(lim < 0 ? 0 : lim);
  const bool reaches_chunk = fused && lim >= len_prev;
  k.chunk_row0 = reaches_chunk ? (unsigned)len_prev : 0xffffffffu;
  k.t_new = reaches_chunk ? (int)((len_prev + kTileKeys - 1) / kTileKeys) : 0x7fffffff;
  k.t_straddle = reaches_chunk && len_prev % kTileKeys ? (int)(len_prev / kTileKeys) : -1;
  return k;
}

// Source of ring row `row_in_tile` (0 .. 63) of physical tile t_phys: a cache row of the KV head, or a row of the
// chunk as handed in (counted from its first row), clamped as described above.
struct DmaRow {
  bool from_chunk;
  unsigned row;
};
KVFOLD_HD DmaRow dma_row(const KeyRange& k, int t_phys, int row_in_tile) {
  unsigned r = (unsigned)(t_phys * kTileKeys + row_in_tile);
  r = r < k.row_lim ? r : k.row_lim;
  DmaRow d;
  d.from_chunk = r >= k.chunk_row0;
  d.row = d.from_chunk ? r - k.chunk_row0 : r;
  return d;
}

}  // namespace kvfold
