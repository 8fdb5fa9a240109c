// Chunk-prefix attention of the fold step, bf16 operands on the gfx950 matrix cores.
//
// What it computes (paper Sec. 2, "KV-Fold"): row i of the chunk, query head h, attends to cache
// rows j <= len_prev + i of KV head h / G -- the whole prefix plus the causal part of the chunk
// itself, whose rows the append kernel has already written:
//     out[i][h] = sum_j softmax_j(scale * q[i][h] . K[j]) V[j].
//
// Mapping to the machine
//  * Work unit = (32 consecutive chunk rows, one query head).  A wavefront owns QB units, a
//    workgroup 4 wavefronts; all units of a workgroup share one KV head, so a K/V tile staged in
//    LDS is reused across the grouped-query heads.  Units are ordered token-block-major, head-minor,
//    so the wavefronts of a workgroup see (almost) the same key range and only the last tiles
//    need the causal mask.
//  * Per 64-key tile a wavefront forms S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (keys are the M
//    rows), so each lane ends up with 32 logits of ONE query: row max / row sum are in-lane plus a
//    single exchange between lanes l and l^32.  The accumulator layout of S^T is, up to a fixed
//    permutation of the keys inside a 16-key slab, the B-operand layout of the next product
//    O^T = V^T P^T; V^T fragments are read from the row-major V tile with the LDS transpose read
//    (ds_read_b64_tr_b16) using the same permutation, so P never leaves registers.
//  * Online softmax in base 2 (scale*log2 e folded into one FMA), running max kept stale until it
//    grows by more than 2^8 (then O and l are rescaled), P rounded to bf16 by the hardware pack
//    convert, row sums accumulated from the ROUNDED values so weights stay a convex combination.
//  * Optional split of the key range over workgroups: partial (max, sum, O) go to a workspace
//    and are merged by the combine kernel.
#include "kvfold_internal.h"

namespace kvfold {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short short4_;
typedef __attribute__((ext_vector_type(8))) short short8_;
typedef __attribute__((ext_vector_type(16))) float floatx16;

#define LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

__device__ __forceinline__ float pair_max(float x) {
  // lanes l and l^32 exchange x; both end with the maximum
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

constexpr float kRescaleThreshold = 8.0f;  // log2 units: stale running max tolerated up to 2^8

template <int D, int QB>
__global__ void __launch_bounds__(256, (QB == 1 ? 2 : 1)) attn_bf16_kernel(AttnParams p) {
  constexpr int CH = D / 8;         // 16-byte chunks per row
  constexpr int ROWB = D * 2;       // bytes per row
  constexpr int BN = kTileKeys;     // 64
  constexpr int KS = D / 16;        // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;        // 32-wide blocks of the head dim in O^T
  constexpr int LD_IT = BN * CH / 256;
  constexpr int KSW = CH < 16 ? CH : 16;  // K swizzle period (rows)
  constexpr int VSW = CH / 4;             // V swizzle: chunk ^= (row & 3) * VSW

  __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BN * ROWB];
  unsigned char* sK = smem;
  unsigned char* sV = smem + BN * ROWB;

  // ---- which workgroup am I (XCD-aware: contiguous logical ranges per XCD)
  const int per_xcd = gridDim.x / kNumXcd;
  const int lid = (blockIdx.x % kNumXcd) * per_xcd + blockIdx.x / kNumXcd;
  if (lid >= p.n_wgs) return;
  const int wgs_per_kvh = p.wgs_per_head * p.n_splits;
  const int g = lid / wgs_per_kvh;
  const int rem = lid - g * wgs_per_kvh;
  const int split = rem / p.wgs_per_head;
  const int ug = p.wgs_per_head - 1 - (rem - split * p.wgs_per_head);  // heaviest (latest rows) first

  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, hi = l >> 5, m = l & 31;
  const int C = p.n_tokens, Hq = p.n_q_heads, G = p.group;
  const int64_t L = p.len_prev + C;
  constexpr int UPW = kUnitsPerWg * QB;  // units per workgroup

  // ---- my units: Q fragments stay in registers for the whole kernel
  bf16x8 qf[QB][KS];
  int tok[QB], head[QB];
  bool store_ok[QB];
  int64_t my_vis[QB];     // keys visible to this lane's query row
  int64_t vis_first[QB];  // keys visible to the unit's first row (tiles below need no mask)
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int u = (ug * kUnitsPerWg + w) * QB + qb;
    const int uc = u < p.units_per_head ? u : p.units_per_head - 1;
    const int tb = uc / G, hg = uc - tb * G;
    head[qb] = g * G + hg;
    tok[qb] = tb * kRowsPerUnit + m;
    const int tokc = tok[qb] < C ? tok[qb] : C - 1;
    store_ok[qb] = (u < p.units_per_head) && (tok[qb] < C);
    my_vis[qb] = p.len_prev + tokc + 1;
    vis_first[qb] = p.len_prev + (int64_t)tb * kRowsPerUnit + 1;
    const __bf16* qrow = reinterpret_cast<const __bf16*>(p.q) + ((int64_t)tokc * Hq + head[qb]) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16 + hi * 8);
  }

  // ---- tile range of this workgroup / split
  int64_t nkeys_wg;
  {
    int ulast = ug * UPW + UPW - 1;
    if (ulast > p.units_per_head - 1) ulast = p.units_per_head - 1;
    int row_hi = (ulast / G) * kRowsPerUnit + kRowsPerUnit - 1;
    if (row_hi > C - 1) row_hi = C - 1;
    nkeys_wg = p.len_prev + row_hi + 1;
  }
  const int ntiles = (int)((nkeys_wg + BN - 1) / BN);
  const int t_begin = split * p.tiles_per_split;
  int t_end = t_begin + p.tiles_per_split;
  if (t_end > ntiles) t_end = ntiles;

  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k_cache) + (int64_t)g * p.capacity * ROWB;
  const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v_cache) + (int64_t)g * p.capacity * ROWB;

  // ---- per-thread staging slots: chunk ci = it*256 + tid of the tile
  uint4 kreg[LD_IT], vreg[LD_IT];
  int ld_row[LD_IT], ld_koff[LD_IT], ld_voff[LD_IT], ld_goff[LD_IT];
#pragma unroll
  for (int it = 0; it < LD_IT; ++it) {
    const int ci = it * 256 + tid;
    const int row = ci / CH, c = ci % CH;
    ld_row[it] = row;
    ld_goff[it] = c * 16;
    ld_koff[it] = row * ROWB + ((c ^ (row % KSW)) * 16);
    ld_voff[it] = row * ROWB + ((c ^ ((row & 3) * VSW)) * 16);
  }
  auto load_tile = [&](int t) {
#pragma unroll
    for (int it = 0; it < LD_IT; ++it) {
      int64_t grow = (int64_t)t * BN + ld_row[it];
      if (grow > L - 1) grow = L - 1;  // rows past the cache end are masked anyway; never read them
      kreg[it] = *reinterpret_cast<const uint4*>(kbase + grow * ROWB + ld_goff[it]);
      vreg[it] = *reinterpret_cast<const uint4*>(vbase + grow * ROWB + ld_goff[it]);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int it = 0; it < LD_IT; ++it) {
      *reinterpret_cast<uint4*>(sK + ld_koff[it]) = kreg[it];
      *reinterpret_cast<uint4*>(sV + ld_voff[it]) = vreg[it];
    }
  };

  // ---- LDS read addresses
  // K fragment (A operand of S^T): row kb*32+m, chunk ks*2+hi (swizzled by row % KSW = m % KSW)
  const int k_row_off = m * ROWB;
  const int k_sw = m % KSW;
  // V^T fragment via transpose read: lane i of a 16-lane block supplies row (i/4), 4 columns
  const int i16 = l & 15, b2 = (l >> 4) & 1;
  const int v_row = 4 * hi + (i16 >> 2);                       // + 16*t (+8)
  const int v_chunk_lo = 2 * b2 + ((i16 & 3) >> 1);           // + 4*db, then swizzled
  const int v_inner = 8 * (i16 & 1);
  const int v_sw = (v_row & 3) * VSW;

  // ---- running state
  floatx16 o[QB][DB];
  float m_run[QB], l_run[QB];
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    m_run[qb] = -INFINITY;
    l_run[qb] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
  }
  const float sc = p.scale_log2e;

  if (t_begin < t_end) load_tile(t_begin);
  for (int t = t_begin; t < t_end; ++t) {
    __syncthreads();  // everyone finished reading the previous tile
    store_tile();
    __syncthreads();
    if (t + 1 < t_end) load_tile(t + 1);  // in flight while this tile is consumed

    // ---- S^T = K Q^T
    floatx16 s[QB][2];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[qb][kb][r] = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 a =
            *reinterpret_cast<const bf16x8*>(sK + kb * 32 * ROWB + k_row_off + (((ks * 2 + hi) ^ k_sw) * 16));
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) s[qb][kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[qb][kb], 0, 0, 0);
      }
    }

    // ---- online softmax (per lane: one query, 32 keys)
    bf16x8 pb[QB][4];
    const int64_t tile_key0 = (int64_t)t * BN;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const bool need_mask = tile_key0 + BN > vis_first[qb];  // wave-uniform
      if (need_mask) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int64_t j = tile_key0 + kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
            if (j >= my_vis[qb]) s[qb][kb][r] = -INFINITY;
          }
      }
      float mx = s[qb][0][0];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[qb][kb][r]);
      mx = pair_max(mx) * sc;  // sc > 0, so the max commutes with the scaling
      if (__any(mx > m_run[qb] + kRescaleThreshold)) {
        const float m2 = fmaxf(m_run[qb], mx);
        const float alpha = (m2 == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(m_run[qb] - m2);
        m_run[qb] = m2;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
      }
      const float m_use = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
      bf16x2 ones;
      ones[0] = (__bf16)1.0f;
      ones[1] = (__bf16)1.0f;
      float lsum = 0.f;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(s[qb][kb][r], sc, -m_use));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(s[qb][kb][r + 1], sc, -m_use));
          bf16x2 pk;
          pk[0] = (__bf16)p0;
          pk[1] = (__bf16)p1;
          lsum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, lsum, false);
          const int tt = kb * 2 + (r >> 3), e = r & 7;
          pb[qb][tt][e] = pk[0];
          pb[qb][tt][e + 1] = pk[1];
        }
      l_run[qb] += lsum;
    }

    // ---- O^T += V^T P^T
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const unsigned char* a0 =
            sV + (16 * tt + v_row) * ROWB + (((4 * db + v_chunk_lo) ^ v_sw) * 16) + v_inner;
        const short4_ lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4_, a0));
        const short4_ hi4 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4_, a0 + 8 * ROWB));
        const short8_ a8 = __builtin_shufflevector(lo, hi4, 0, 1, 2, 3, 4, 5, 6, 7);
        const bf16x8 a = __builtin_bit_cast(bf16x8, a8);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) o[qb][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb[qb][tt], o[qb][db], 0, 0, 0);
      }
    }
  }

  // ---- epilogue
  const int64_t n_rows = (int64_t)C * Hq;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = pair_sum(l_run[qb]);
    if (!store_ok[qb]) continue;
    const int64_t row = (int64_t)tok[qb] * Hq + head[qb];
    if (p.n_splits == 1) {
      const float inv = 1.f / l_tot;
      __bf16* orow = reinterpret_cast<__bf16*>(p.out) + row * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[qb][db][rg * 4 + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + db * 32 + 8 * rg + 4 * hi) = v;
        }
      if (p.lse && hi == 0)
        p.lse[(int64_t)head[qb] * C + tok[qb]] = (m_run[qb] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
    } else {
      float* prow = p.part_o + ((int64_t)split * n_rows + row) * D;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          float4 v = make_float4(o[qb][db][rg * 4 + 0], o[qb][db][rg * 4 + 1], o[qb][db][rg * 4 + 2],
                                 o[qb][db][rg * 4 + 3]);
          *reinterpret_cast<float4*>(prow + db * 32 + 8 * rg + 4 * hi) = v;
        }
      if (hi == 0) {
        float2 ml = make_float2(m_run[qb], l_tot);
        *reinterpret_cast<float2*>(p.part_ml + ((int64_t)split * n_rows + row) * 2) = ml;
      }
    }
  }
}

template <int D, int QB>
static hipError_t launch_one(const AttnParams& p, hipStream_t s) {
  hipLaunchKernelGGL((attn_bf16_kernel<D, QB>), dim3(padded_grid(p.n_wgs)), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_attn_bf16(const AttnParams& p, int head_dim, int qb, hipStream_t s) {
  if (head_dim == 128) return qb == 2 ? launch_one<128, 2>(p, s) : launch_one<128, 1>(p, s);
  if (head_dim == 64) return qb == 2 ? launch_one<64, 2>(p, s) : launch_one<64, 1>(p, s);
  return hipErrorInvalidValue;
}

}  // namespace kvfold
