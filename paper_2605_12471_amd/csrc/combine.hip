// Merge of split-prefix partial results.  When a chunk has too few rows to fill the chip, the key
// range of one fold step (paper Sec. 2: keys K_{0:t}) is cut into S contiguous pieces handled by
// different workgroups; each leaves, per (row, head), its running maximum m_s (log2 units), the
// sum l_s of 2^(logit - m_s) and the unnormalised O_s.  Softmax over the union is recovered exactly:
//   M = max_s m_s,  L = sum_s l_s 2^(m_s - M),  out = sum_s O_s 2^(m_s - M) / L.
// HBM-bound (reads S * (d + 2) floats per row once, writes d elements); launch-latency bound for few rows.
#include "kvfold_internal.h"

namespace kvfold {

// Thread layout of a 256-thread block: rows_per_block rows x SG split groups x V 16-byte column
// vectors (V = head_dim / 4).  Split group sg of a row folds pieces sg, sg + SG, ... into one running
// (m, l, O); the SG results meet in LDS.  With few rows (decode-shaped steps: 32 rows, 64 pieces) this
// keeps every load of a row in flight at once instead of walking the pieces one after another.
constexpr int kCombineThreads = 256;

__global__ void __launch_bounds__(kCombineThreads) combine_kernel(CombineParams p, int SG, int rows_per_block) {
  extern __shared__ float4 red[];  // [rows_per_block][SG][V] partial O, then [rows_per_block][SG] (m, l) pairs
  const int V = p.head_dim >> 2;
  const int tid = threadIdx.x;
  const int dv = tid % V, sg = (tid / V) % SG, rl = tid / (V * SG);
  const int64_t row = (int64_t)blockIdx.x * rows_per_block + rl;
  const bool live = rl < rows_per_block && row < p.n_rows;
  float2* red_ml = reinterpret_cast<float2*>(red + rows_per_block * SG * V);

  float m = -INFINITY, l = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  if (live) {
    // pieces in batches of kBatch: all loads of a batch are in flight before the first is folded in
    constexpr int kBatch = 4;
    for (int s0 = sg; s0 < p.n_splits; s0 += SG * kBatch) {
      float2 ml[kBatch];
      float4 o[kBatch];
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        const int s = s0 + u * SG;
        if (s < p.n_splits) {
          ml[u] = *reinterpret_cast<const float2*>(p.part_ml + ((int64_t)s * p.n_rows + row) * 2);
          o[u] = *reinterpret_cast<const float4*>(p.part_o + ((int64_t)s * p.n_rows + row) * p.head_dim + dv * 4);
        } else {
          ml[u] = make_float2(0.f, 0.f);
          o[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
#pragma unroll
      for (int u = 0; u < kBatch; ++u) {
        if (ml[u].y == 0.f) continue;  // this piece saw no visible key for the row (or lies past the last piece)
        const float mn = fmaxf(m, ml[u].x);
        const float a = exp2f(m - mn), b = exp2f(ml[u].x - mn);  // m = -inf the first time: a = 0
        l = l * a + ml[u].y * b;
        acc.x = acc.x * a + o[u].x * b;
        acc.y = acc.y * a + o[u].y * b;
        acc.z = acc.z * a + o[u].z * b;
        acc.w = acc.w * a + o[u].w * b;
        m = mn;
      }
    }
    red[(rl * SG + sg) * V + dv] = acc;
    if (dv == 0) red_ml[rl * SG + sg] = make_float2(m, l);
  }
  __syncthreads();
  if (!live || sg != 0) return;

  float M = -INFINITY;
  for (int g = 0; g < SG; ++g) M = fmaxf(M, red_ml[rl * SG + g].x);
  float Lsum = 0.f;
  acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int g = 0; g < SG; ++g) {
    const float2 ml = red_ml[rl * SG + g];
    if (ml.y == 0.f) continue;
    const float wgt = exp2f(ml.x - M);
    Lsum += wgt * ml.y;
    const float4 o = red[(rl * SG + g) * V + dv];
    acc.x += wgt * o.x;
    acc.y += wgt * o.y;
    acc.z += wgt * o.z;
    acc.w += wgt * o.w;
  }
  const float inv = 1.f / Lsum;
  acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  if (p.out_is_bf16) {
    typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
    bf16x4 v;
    v[0] = (__bf16)acc.x; v[1] = (__bf16)acc.y; v[2] = (__bf16)acc.z; v[3] = (__bf16)acc.w;
    *reinterpret_cast<bf16x4*>(reinterpret_cast<__bf16*>(p.out) + row * p.head_dim + dv * 4) = v;
  } else {
    *reinterpret_cast<float4*>(reinterpret_cast<float*>(p.out) + row * p.head_dim + dv * 4) = acc;
  }
  if (p.lse && dv == 0) {
    const int64_t tok = row / p.n_q_heads;
    const int64_t head = row - tok * p.n_q_heads;
    p.lse[head * p.n_tokens + tok] = (M + log2f(Lsum)) * 0.6931471805599453f;
  }
}

hipError_t launch_combine(const CombineParams& p, hipStream_t s) {
  if (p.n_rows <= 0) return hipSuccess;
  const int V = p.head_dim >> 2;  // 16 or 32
  // Split groups (a power of two, at most the number of pieces and what one row's share of a block
  // allows) only as far as they are needed to put about two blocks on every CU: with many rows one
  // thread per (row, column vector) walking the pieces is the cheaper form.
  const int64_t blocks1 = ((int64_t)p.n_rows * V + kCombineThreads - 1) / kCombineThreads;
  int SG = 1;
  while (SG < p.n_splits && SG * 2 * V <= kCombineThreads && blocks1 * SG < 512) SG *= 2;
  const int rows_per_block = kCombineThreads / (V * SG);
  const unsigned blocks = (unsigned)((p.n_rows + rows_per_block - 1) / rows_per_block);
  const size_t lds = (size_t)rows_per_block * SG * (V * sizeof(float4) + sizeof(float2));
  hipLaunchKernelGGL(combine_kernel, dim3(blocks), dim3(kCombineThreads), lds, s, p, SG, rows_per_block);
  return hipGetLastError();
}

}  // namespace kvfold
