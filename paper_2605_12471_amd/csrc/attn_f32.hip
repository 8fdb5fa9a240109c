// Chunk-prefix attention of the fold step in fp32 throughout (the precision-ablation mode of the
// paper's Sec. 3; here the 1e-5 correctness mode).  Same decomposition as the bf16 kernel: a
// wavefront owns one (32 chunk rows, one query head) unit, 4 wavefronts of one KV head share
// each 64-key K/V tile through LDS, logits are formed transposed (S^T = K Q^T, keys as MFMA rows)
// with v_mfma_f32_32x32x2_f32 so a lane holds 32 logits of one query, and the accumulator layout
// of S^T feeds O^T = V^T P^T directly: register r of S^T pairs the two keys 8*(r/4) + r%4 and
// that + 4 held by the two half-waves, which are exactly the K=2 contraction slots of the MFMA.
#include "kvfold_internal.h"

namespace kvfold {

typedef __attribute__((ext_vector_type(16))) float floatx16;

__device__ __forceinline__ float pair_max_f(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum_f(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <int D, bool WIN>  // WIN: the sink + sliding-window step
__global__ void __launch_bounds__(256, 2) attn_f32_kernel(AttnParams p) {
  constexpr int CH = D / 4;    // 16-byte chunks per row
  constexpr int ROWB = D * 4;  // bytes per row
  constexpr int BN = kTileKeys;
  constexpr int DB = D / 32;
  constexpr int LD_IT = BN * CH / 256;
  constexpr float kThresh = 8.0f;

  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BN * ROWB];
  unsigned char* sK = smem;
  unsigned char* sV = smem + BN * ROWB;

  const int wgs_per_kvh = p.wgs_per_head * p.n_splits;
  const int lid = logical_workgroup((int)blockIdx.x, (int)gridDim.x, p.n_q_heads / p.group, wgs_per_kvh);
  if (lid >= p.n_wgs) return;
  const int g = lid / wgs_per_kvh;
  const int rem = lid - g * wgs_per_kvh;
  const int split = rem / p.wgs_per_head;
  // Later token blocks see more keys.  Default order: heaviest first (longest-processing-time
  // first over several rounds of workgroups).  With pair_order the grid is resident at once, two
  // workgroups per CU, dispatched in id order: the first half descends from the heaviest, the second
  // half ascends from the lightest, so the two workgroups that share a CU add up to the same work.
  int ug;
  {
    const int idx = rem - split * p.wgs_per_head, W = p.wgs_per_head, half = (W + 1) / 2;
    ug = (!p.pair_order || idx < half) ? W - 1 - idx : idx - half;
  }

  const int tid = threadIdx.x, l = tid & 63, hi = l >> 5, m = l & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: what depends on it alone stays in scalar registers
  const int C = p.n_tokens, Hq = p.n_q_heads, G = p.group;
  const int L = (int)p.len_prev + C;  // (row counts fit 32 bits: the host limits the capacity to 2^30 rows)

  const int u = ug * kUnitsPerWg + w;
  const int uc = u < p.units_per_head ? u : p.units_per_head - 1;
  const int tb = uc / G, hg = uc - tb * G;
  const int head = g * G + hg;
  const int tok = tb * kRowsPerUnit + m;
  const int tokc = tok < C ? tok : C - 1;
  const bool store_ok = (u < p.units_per_head) && (tok < C);
  const int my_vis = (int)p.len_prev + tokc + 1;
  const int vis_first = (int)p.len_prev + tb * kRowsPerUnit + 1;
  // Sink + sliding-window step (Sec. 6 of the paper, the streaming baseline's mask): of the keys [0, vis) a row
  // sees only j < n_sink and j >= vis - window; lb_last is the largest such lower bound among the unit's rows
  constexpr bool win = WIN;
  int lb_last;
  {
    const int last = tb * kRowsPerUnit + kRowsPerUnit - 1;
    lb_last = (int)p.len_prev + (last < C ? last : C - 1) + 1 - p.window;
  }

  // Q: lane (m, hi) keeps q[m][8*s + 4*hi + j], j = 0..3, s = 0..D/8-1 (contraction slot hi of MFMA (s,j))
  float4 qf[D / 8];
  {
    const float* qrow = reinterpret_cast<const float*>(p.q) + ((int64_t)tokc * Hq + head) * D;
#pragma unroll
    for (int s8 = 0; s8 < D / 8; ++s8) {
      float4 v = *reinterpret_cast<const float4*>(qrow + s8 * 8 + hi * 4);
      if (p.rope_cos) {
        // Rotary embedding at the row's absolute position (Sec. 2), half-split pairs (j, j + D/2): the sine
        // product rounded first, then one fused multiply-add
        const bool lower = s8 < D / 16;
        const int j0 = (lower ? s8 : s8 - D / 16) * 8 + hi * 4;  // index of the pair's angle
        const float4 o = *reinterpret_cast<const float4*>(qrow + (lower ? D / 2 : 0) + j0);
        const float4 cs = *reinterpret_cast<const float4*>(p.rope_cos + (int64_t)tokc * (D / 2) + j0);
        const float4 sn = *reinterpret_cast<const float4*>(p.rope_sin + (int64_t)tokc * (D / 2) + j0);
        const float tx = o.x * sn.x, ty = o.y * sn.y, tz = o.z * sn.z, tw = o.w * sn.w;
        v.x = __builtin_fmaf(v.x, cs.x, lower ? -tx : tx);
        v.y = __builtin_fmaf(v.y, cs.y, lower ? -ty : ty);
        v.z = __builtin_fmaf(v.z, cs.z, lower ? -tz : tz);
        v.w = __builtin_fmaf(v.w, cs.w, lower ? -tw : tw);
      }
      qf[s8] = v;
    }
  }

  int nkeys_wg;
  {
    int ulast = ug * kUnitsPerWg + kUnitsPerWg - 1;
    if (ulast > p.units_per_head - 1) ulast = p.units_per_head - 1;
    int row_hi = (ulast / G) * kRowsPerUnit + kRowsPerUnit - 1;
    if (row_hi > C - 1) row_hi = C - 1;
    nkeys_wg = (int)p.len_prev + row_hi + 1;
  }
  // logical tiles 0 .. ntiles-1; under a window the tiles between the sinks and the window are left out:
  // logical tile t is physical tile t + (t >= ns_t ? skip : 0)
  TileMap tm;
  if (win) {
    const RowRange rr = workgroup_rows(ug, kUnitsPerWg, p.units_per_head, G, C);
    tm = tile_map(p.len_prev, rr.row_lo, rr.row_hi, p.n_sink, p.window);
  } else {
    tm.ns_t = 0;
    tm.skip = 0;
    tm.ntiles = (nkeys_wg + BN - 1) / BN;
  }
  const int ntiles = tm.ntiles;
  const int t_begin = split * p.tiles_per_split;
  int t_end = t_begin + p.tiles_per_split;
  if (t_end > ntiles) t_end = ntiles;

  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k_cache) + (int64_t)g * p.capacity * ROWB;
  const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v_cache) + (int64_t)g * p.capacity * ROWB;

  // K tile: chunk c of row r stored at chunk c ^ (r % 16)  (16 lanes with consecutive rows, one column -> 16 banksets)
  // V tile: chunk c of row r stored at chunk c ^ (8 * ((r >> 2) & 1))  (rows r and r+4 read together by the half-waves)
  floatx16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) o[db][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float sc = p.scale_log2e;

  for (int t_log = t_begin; t_log < t_end; ++t_log) {
    const int t = t_log + (t_log >= tm.ns_t ? tm.skip : 0);
    __syncthreads();
#pragma unroll
    for (int it = 0; it < LD_IT; ++it) {
      const int ci = it * 256 + tid;
      const int row = ci / CH, c = ci % CH;
      int grow = t * BN + row;
      if (grow > L - 1) grow = L - 1;
      const uint4 kv = *reinterpret_cast<const uint4*>(kbase + (int64_t)grow * ROWB + c * 16);
      const uint4 vv = *reinterpret_cast<const uint4*>(vbase + (int64_t)grow * ROWB + c * 16);
      *reinterpret_cast<uint4*>(sK + row * ROWB + ((c ^ (row & 15)) * 16)) = kv;
      *reinterpret_cast<uint4*>(sV + row * ROWB + ((c ^ (8 * ((row >> 2) & 1))) * 16)) = vv;
    }
    __syncthreads();

    // ---- S^T = K Q^T
    floatx16 s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
      const int row = kb * 32 + m;
#pragma unroll
      for (int s8 = 0; s8 < D / 8; ++s8) {
        const int c = s8 * 2 + hi;
        const float4 a = *reinterpret_cast<const float4*>(sK + row * ROWB + ((c ^ (row & 15)) * 16));
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, qf[s8].x, s[kb], 0, 0, 0);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, qf[s8].y, s[kb], 0, 0, 0);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, qf[s8].z, s[kb], 0, 0, 0);
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, qf[s8].w, s[kb], 0, 0, 0);
      }
    }

    // ---- online softmax
    const int tile_key0 = t * BN;
    const bool left = WIN && tile_key0 < lb_last && tile_key0 + BN > p.n_sink;  // keys between the sinks and the window
    if (tile_key0 + BN > vis_first || left) {
      // visible inside the tile: keys below rel, and of those (window step) the ones below rel_sink or from rel_lb
      // on; all three are counted from the lane's own first key, 4 * hi
      // (opaque copy of the lane's half: the 32 key offsets below are formed here, not once ahead of the tile loop
      // and then held in registers through it)
      int hi_here = hi;
      asm volatile("" : "+v"(hi_here));
      const int rel = my_vis - tile_key0 - 4 * hi_here;
      const int rel_lb = WIN ? rel - p.window : -1, rel_sink = WIN ? p.n_sink - tile_key0 - 4 * hi_here : 0;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kk = kb * 32 + 8 * (r >> 2) + (r & 3);  // key offset in the tile, less the lane's 4 * hi
          if (kk >= rel || (WIN && kk < rel_lb && kk >= rel_sink)) s[kb][r] = -INFINITY;
        }
    }
    float mx = s[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    mx = pair_max_f(mx) * sc;
    if (__any(mx > m_run + kThresh)) {
      // only rows that asked for it move, so a row's arithmetic never depends on its wave neighbours
      const float m2 = (mx > m_run + kThresh) ? mx : m_run;
      const float alpha = (m2 == -INFINITY) ? 1.f : exp2f(m_run - m2);
      m_run = m2;
      l_run *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
    }
    const float m_use = (m_run == -INFINITY) ? 0.f : m_run;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        s[kb][r] = exp2f(fmaf(s[kb][r], sc, -m_use));
        l_run += s[kb][r];
      }

    // ---- O^T += V^T P^T : register r of block kb contracts keys kb*32 + 8*(r/4) + r%4 (+4 for hi = 1)
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = kb * 32 + 8 * (r >> 2) + (r & 3) + 4 * hi;
        const int sw = 8 * ((row >> 2) & 1);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int col = db * 32 + m;  // float column
          const int c = (col >> 2) ^ sw;
          const float a = *reinterpret_cast<const float*>(sV + row * ROWB + c * 16 + (col & 3) * 4);
          o[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, s[kb][r], o[db], 0, 0, 0);
        }
      }
  }

  // ---- epilogue
  const float l_tot = pair_sum_f(l_run);
  if (!store_ok) return;
  const int64_t n_rows = (int64_t)C * Hq;
  const int64_t row = (int64_t)tok * Hq + head;
  if (p.n_splits == 1) {
    const float inv = 1.f / l_tot;
    float* orow = reinterpret_cast<float*>(p.out) + row * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg)
        *reinterpret_cast<float4*>(orow + db * 32 + 8 * rg + 4 * hi) =
            make_float4(o[db][rg * 4 + 0] * inv, o[db][rg * 4 + 1] * inv, o[db][rg * 4 + 2] * inv, o[db][rg * 4 + 3] * inv);
    if (p.lse && hi == 0) p.lse[(int64_t)head * C + tok] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
  } else {
    float* prow = p.part_o + ((int64_t)split * n_rows + row) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg)
        *reinterpret_cast<float4*>(prow + db * 32 + 8 * rg + 4 * hi) =
            make_float4(o[db][rg * 4 + 0], o[db][rg * 4 + 1], o[db][rg * 4 + 2], o[db][rg * 4 + 3]);
    if (hi == 0) *reinterpret_cast<float2*>(p.part_ml + ((int64_t)split * n_rows + row) * 2) = make_float2(m_run, l_tot);
  }
}

hipError_t launch_attn_f32(const AttnParams& p, int head_dim, hipStream_t s) {
  const dim3 grid(padded_grid(p.n_wgs));
  if (head_dim == 128 && p.window > 0)
    hipLaunchKernelGGL((attn_f32_kernel<128, true>), grid, dim3(256), 0, s, p);
  else if (head_dim == 128)
    hipLaunchKernelGGL((attn_f32_kernel<128, false>), grid, dim3(256), 0, s, p);
  else if (head_dim == 64 && p.window > 0)
    hipLaunchKernelGGL((attn_f32_kernel<64, true>), grid, dim3(256), 0, s, p);
  else if (head_dim == 64)
    hipLaunchKernelGGL((attn_f32_kernel<64, false>), grid, dim3(256), 0, s, p);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace kvfold
