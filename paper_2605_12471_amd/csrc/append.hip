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

// The same carry with the rotary embedding applied to the K rows on the way (Sec. 2: the new tokens'
// positions continue from the absolute position, so their rotations line up with the original
// sequence).  Element j pairs with element j + d/2 (half-split layout):
//     k'_j = k_j cos_j - k_{j+d/2} sin_j,   k'_{j+d/2} = k_{j+d/2} cos_j + k_j sin_j,
// in fp32 -- the product of the other element with the sine rounded first, then one fused
// multiply-add -- and rounded to the cache's element type (RNE).  A lane owns 16 bytes of a row and
// reads the 16 bytes half a row away as well.  V rows are copied bit for bit.
template <typename T, int E>  // element type, elements per 16-byte vector
__global__ void __launch_bounds__(256) append_rope_kernel(AppendParams p) {
  typedef __attribute__((ext_vector_type(E))) T vec_t;
  const bool is_v = blockIdx.y != 0;
  const vec_t* __restrict__ src = reinterpret_cast<const vec_t*>(is_v ? p.v_new : p.k_new);
  vec_t* __restrict__ dst = reinterpret_cast<vec_t*>(is_v ? p.v_cache : p.k_cache);
  const int64_t vec_per_row = p.row_bytes >> 4;
  const int64_t half_vecs = vec_per_row >> 1;
  const int64_t half_d = half_vecs * E;
  const int64_t per_head = (int64_t)p.n_tokens * vec_per_row;
  const int64_t total = per_head * p.n_kv_heads;
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
       idx += (int64_t)gridDim.x * blockDim.x) {
    const int64_t g = idx / per_head;
    const int64_t rem = idx - g * per_head;
    const int64_t i = rem / vec_per_row;
    const int64_t c = rem - i * vec_per_row;
    const vec_t* row = src + (i * p.n_kv_heads + g) * vec_per_row;
    vec_t v = row[c];
    if (!is_v) {
      const bool lower = c < half_vecs;
      const vec_t other = row[lower ? c + half_vecs : c - half_vecs];
      const float* cs = p.rope_cos + i * half_d + (lower ? c : c - half_vecs) * E;
      const float* sn = p.rope_sin + i * half_d + (lower ? c : c - half_vecs) * E;
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const float mine = (float)v[e], theirs = (float)other[e];
        const float t = theirs * sn[e];
        v[e] = (T)__builtin_fmaf(mine, cs[e], lower ? -t : t);
      }
    }
    dst[(g * p.capacity + p.len_prev + i) * vec_per_row + c] = v;
  }
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
  const int64_t total = (int64_t)p.n_tokens * p.n_kv_heads * (p.row_bytes >> 4);
  if (total <= 0) return hipSuccess;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (!p.rope_cos)
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, s, p);
  else if (p.elem_is_bf16)
    hipLaunchKernelGGL((append_rope_kernel<__bf16, 8>), dim3((unsigned)blocks, 2), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((append_rope_kernel<float, 4>), dim3((unsigned)blocks, 2), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace kvfold
