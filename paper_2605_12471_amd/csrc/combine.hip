// Merge of split-prefix partial results.  When a chunk has too few rows to fill the chip, the key
// range of one fold step (paper Sec. 2: keys K_{0:t}) is cut into S contiguous pieces handled by
// different workgroups; each leaves, per (row, head), its running maximum m_s (log2 units), the
// sum l_s of 2^(logit - m_s) and the unnormalised O_s.  Softmax over the union is recovered exactly:
//   M = max_s m_s,  L = sum_s l_s 2^(m_s - M),  out = sum_s O_s 2^(m_s - M) / L.
// HBM-bound (reads S * (d + 2) floats per row once, writes d elements).
#include "kvfold_internal.h"

namespace kvfold {

__global__ void __launch_bounds__(256) combine_kernel(CombineParams p) {
  const int vec_per_row = p.head_dim >> 2;
  const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int64_t row = gid / vec_per_row;
  const int dv = (int)(gid - row * vec_per_row);
  if (row >= p.n_rows) return;

  float M = -INFINITY;
  for (int s = 0; s < p.n_splits; ++s) M = fmaxf(M, p.part_ml[((int64_t)s * p.n_rows + row) * 2]);
  float Lsum = 0.f;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < p.n_splits; ++s) {
    const float2 ml = *reinterpret_cast<const float2*>(p.part_ml + ((int64_t)s * p.n_rows + row) * 2);
    if (ml.y == 0.f) continue;  // this piece saw no visible key for the row
    const float wgt = exp2f(ml.x - M);
    Lsum += wgt * ml.y;
    const float4 o = *reinterpret_cast<const float4*>(p.part_o + ((int64_t)s * p.n_rows + row) * p.head_dim + dv * 4);
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
  const int64_t threads = (int64_t)p.n_rows * (p.head_dim >> 2);
  if (threads <= 0) return hipSuccess;
  hipLaunchKernelGGL(combine_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace kvfold
