// Cache carry of the fold step (paper Sec. 2 and Fig. 2: the chunk's K/V rows are appended to the
// cache, the prefix is handed on untouched).  Token-major [C][Hkv][d] rows are scattered to the
// head-major cache [Hkv][capacity][d] at rows [len_prev, len_prev + C); a pure bit copy.
//
// HBM-bound: 16 bytes per lane, destination addresses of a wavefront are contiguous (one head's
// rows are adjacent), source addresses are contiguous per row (d * elem_size bytes).
#include "kvfold_internal.h"

namespace kvfold {

__global__ void __launch_bounds__(256) append_kernel(AppendParams p) {
  const bool is_v = blockIdx.y != 0;
  const uint4* __restrict__ src = reinterpret_cast<const uint4*>(is_v ? p.v_new : p.k_new);
  uint4* __restrict__ dst = reinterpret_cast<uint4*>(is_v ? p.v_cache : p.k_cache);
  const int64_t vec_per_row = p.row_bytes >> 4;
  const int64_t per_head = (int64_t)p.n_tokens * vec_per_row;
  const int64_t total = per_head * p.n_kv_heads;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int64_t g = idx / per_head;
    const int64_t rem = idx - g * per_head;
    const int64_t i = rem / vec_per_row;
    const int64_t c = rem - i * vec_per_row;
    dst[(g * p.capacity + p.len_prev + i) * vec_per_row + c] = src[(i * p.n_kv_heads + g) * vec_per_row + c];
  }
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
  const int64_t total = (int64_t)p.n_tokens * p.n_kv_heads * (p.row_bytes >> 4);
  if (total <= 0) return hipSuccess;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(append_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace kvfold
