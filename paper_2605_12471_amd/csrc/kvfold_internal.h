// Internal declarations shared by the HIP translation units of libkvfold (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kvfold_consts.h"
#include "kvfold_plan.h"

namespace kvfold {

struct AppendParams {
  const void* k_new;  // [C][Hkv][d]
  const void* v_new;  // [C][Hkv][d]
  void* k_cache;      // layer base, [Hkv][cap][d]
  void* v_cache;
  int32_t n_tokens;   // C
  int32_t n_kv_heads;
  int32_t row_bytes;  // d * elem_size, multiple of 16
  int64_t capacity;   // rows per head
  int64_t len_prev;   // first destination row
  // Rotary embedding of the K rows on their way into the cache (nullptr: plain bit copy): angles of the
  // rows' absolute positions, [C][d/2] fp32 each; V is never rotated.
  const float* rope_cos;
  const float* rope_sin;
  int32_t elem_is_bf16;
};

struct AttnParams {
  const void* q;         // [C][Hq][d]
  const void* k_cache;   // layer base, [Hkv][cap][d]; rows [0, len_prev + C) valid
  const void* v_cache;
  void* out;             // [C][Hq][d]
  float* lse;            // [Hq][C] or nullptr
  float* part_o;         // [S][C*Hq][d]  unnormalised partial outputs (split mode)
  float* part_ml;        // [S][C*Hq][2]  (running max in log2 units, partial sum)
  int32_t n_tokens;      // C
  int32_t n_q_heads;     // Hq
  int32_t n_kv_heads;    // Hkv
  int32_t group;         // G = Hq / Hkv
  int64_t capacity;      // rows per head in the cache
  int64_t len_prev;      // cache length before this chunk
  int32_t n_splits;      // S >= 1; S == 1 writes out/lse directly
  int32_t tiles_per_split;
  int32_t units_per_head;  // G * ceil(C / 32)
  int32_t wgs_per_head;    // ceil(units_per_head / units per workgroup)
  int32_t n_wgs;           // Hkv * wgs_per_head * S (the grid is padded to a multiple of 8)
  int32_t pair_order;      // 1: every workgroup is resident at once, two per CU; order them heaviest-first for the
                           // first half and lightest-first for the second so each CU gets a balanced pair
  int32_t pair_units;      // two-unit bf16 kernel: a wavefront owns an early and a late unit of the chunk (see the kernel)
  float scale_log2e;       // softmax scale * log2(e)
  // Rotary embedding of the queries as they are loaded (nullptr: q is used as handed in): angles of the
  // chunk's absolute positions, [C][d/2] fp32 each
  const float* rope_cos;
  const float* rope_sin;
  // Append fused into the bf16 attention kernel (nullptr: the cache already holds the chunk's rows): the
  // chunk's K / V rows as handed in, [C][Hkv][d].  Requires len_prev to be a multiple of the 64-key tile, so
  // that a tile lies entirely in the cache or entirely in the chunk.  Tiles of the chunk are then streamed
  // from here, and every workgroup copies its share of the rows into the cache for the steps to come.
  const void* k_new;
  const void* v_new;
  // Sink + sliding-window step (window > 0; 0: every key up to the row's own position is visible): the row at
  // absolute position p sees keys j < n_sink and p - window < j <= p.  Tiles between the sink tiles and the
  // window are skipped (see tile_map()).
  int32_t n_sink;
  int32_t window;
};

struct CombineParams {
  const float* part_o;
  const float* part_ml;
  void* out;
  float* lse;          // [Hq][C] or nullptr
  int32_t n_rows;      // C * Hq
  int32_t n_tokens;    // C
  int32_t n_q_heads;
  int32_t head_dim;
  int32_t n_splits;
  int32_t out_is_bf16;
};

hipError_t launch_append(const AppendParams& p, hipStream_t s);
// In-place storage round trip bf16 -> intN -> bf16 (n_bits = 4 or 8) of cache rows [len_prev, len_prev + C) of K and V.
hipError_t launch_storage_roundtrip(const AppendParams& p, int n_bits, hipStream_t s);
hipError_t launch_attn_bf16(const AttnParams& p, int head_dim, int units_per_wave, hipStream_t s);
// Sets the LDS size attribute of every bf16 attention kernel variant of this head dimension on the current
// device (once per device; launches then have nothing left that could fail for a valid configuration).
hipError_t prepare_attn_bf16(int head_dim);
hipError_t launch_attn_f32(const AttnParams& p, int head_dim, hipStream_t s);
hipError_t launch_combine(const CombineParams& p, hipStream_t s);

// Padded grid size and the XCD-aware remap used by the attention kernels: the hardware hands
// workgroup b to XCD b % 8, so logical ids are dealt out in 8 contiguous ranges, one per XCD,
// which keeps the workgroups of one KV head on one XCD's L2.
inline int padded_grid(int n_wgs) { return (n_wgs + kNumXcd - 1) / kNumXcd * kNumXcd; }
// Logical id (KV head major, then split, then workgroup of the head, heaviest first) of hardware block b.
// A KV head that spans k = 8 / Hkv XCDs has its workgroups dealt to those XCDs in turn, not in k contiguous
// runs: every XCD then gets the same mix of heavy and light workgroups and of prefix splits (a contiguous
// run would put all late token blocks, or a whole split, on one XCD and the light rest on its neighbour).
__device__ __forceinline__ int logical_workgroup(int b, int grid, int n_kv_heads, int wgs_per_kvh) {
  const int x = b % kNumXcd, j = b / kNumXcd;
  if (n_kv_heads < kNumXcd && kNumXcd % n_kv_heads == 0) {
    const int k = kNumXcd / n_kv_heads;
    if (wgs_per_kvh % k == 0) return (x / k) * wgs_per_kvh + j * k + x % k;  // grid = Hkv * wgs_per_kvh, a multiple of 8
  }
  return x * (grid / kNumXcd) + j;
}

}  // namespace kvfold
