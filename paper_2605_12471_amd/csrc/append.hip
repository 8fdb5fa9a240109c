// Cache carry of the fold step (paper Sec. 2 and Fig. 2: the chunk's K/V rows are appended to the
// cache, the prefix is handed on untouched).  Token-major [C][Hkv][d] rows are scattered to the
// head-major cache [Hkv][capacity][d] at rows [len_prev, len_prev + C); a pure bit copy.
//
// HBM-bound: 16 bytes per lane, destination addresses of a wavefront are contiguous (one head's
// rows are adjacent), source addresses are contiguous per row (d * elem_size bytes).
#include "kvfold_internal.h"

namespace kvfold {

// blockIdx.y = 2 * KV head + (0: K, 1: V).  A row is 8, 16 or 32 16-byte vectors (a power of two), so the
// (token, vector) split of an index is a shift and a mask, and one head's destination is one contiguous run.
__global__ void __launch_bounds__(256) append_kernel(AppendParams p, int log2_vpr) {
  const bool is_v = (blockIdx.y & 1) != 0;
  const int64_t g = blockIdx.y >> 1;
  const int64_t vpr = (int64_t)1 << log2_vpr;
  const uint4* __restrict__ src = reinterpret_cast<const uint4*>(is_v ? p.v_new : p.k_new) + g * vpr;
  uint4* __restrict__ dst = reinterpret_cast<uint4*>(is_v ? p.v_cache : p.k_cache) + (g * p.capacity + p.len_prev) * vpr;
  const int64_t per_head = (int64_t)p.n_tokens << log2_vpr;
  const int64_t src_row = (int64_t)p.n_kv_heads << log2_vpr;  // vectors from one token's row to the next
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < per_head; idx += (int64_t)gridDim.x * blockDim.x)
    dst[idx] = src[(idx >> log2_vpr) * src_row + (idx & (vpr - 1))];
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

// Storage perturbation of the carried cache (Sec. 8, Discussion: a per-step quantisation round trip
// bf16 -> intN -> bf16), applied in place to the rows a step has just appended (K and V).  The paper
// names no quantiser; the reading: one group = the d elements of one (token, KV head) row, symmetric,
//   scale = max|x| / (2^(N-1) - 1),  code = round-half-even(x / scale) clamped to +-(2^(N-1) - 1),
//   x' = code * scale,
// all in fp32, stored as bf16 (RNE); an all-zero row stays zero.  A lane owns 16 bytes (8 elements), the
// d / 8 lanes of a row agree on the maximum by butterfly exchanges inside their lane group.
__global__ void __launch_bounds__(256) storage_roundtrip_kernel(AppendParams p, float qmax) {
  typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
  const bool is_v = blockIdx.y != 0;
  bf16x8* __restrict__ cache = reinterpret_cast<bf16x8*>(is_v ? p.v_cache : p.k_cache);
  const int vec_per_row = p.row_bytes >> 4;  // 8 or 16 lanes per row: a power of two, rows never straddle a wavefront
  const int64_t per_head = (int64_t)p.n_tokens * vec_per_row;
  const int64_t total = per_head * p.n_kv_heads;
  const int64_t padded = (total + 255) / 256 * 256;  // whole lane groups stay together through the exchanges
  for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < padded; idx += (int64_t)gridDim.x * blockDim.x) {
    const bool live = idx < total;
    const int64_t cidx = live ? idx : total - 1;
    const int64_t g = cidx / per_head;
    const int64_t rem = cidx - g * per_head;
    const int64_t i = rem / vec_per_row;
    const int64_t c = rem - i * vec_per_row;
    bf16x8* at = cache + (g * p.capacity + p.len_prev + i) * vec_per_row + c;
    bf16x8 v = *at;
    float x[8], amax = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      x[e] = (float)v[e];
      amax = fmaxf(amax, fabsf(x[e]));
    }
    for (int off = 1; off < vec_per_row; off <<= 1) amax = fmaxf(amax, __shfl_xor(amax, off));
    const float scale = amax / qmax;
    if (live && scale > 0.f) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        float code = rintf(x[e] / scale);
        code = fminf(fmaxf(code, -qmax), qmax);
        v[e] = (__bf16)(code * scale);
      }
      *at = v;
    }
  }
}

hipError_t launch_storage_roundtrip(const AppendParams& p, int n_bits, hipStream_t s) {
  const int64_t total = (int64_t)p.n_tokens * p.n_kv_heads * (p.row_bytes >> 4);
  if (total <= 0) return hipSuccess;
  int64_t blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(storage_roundtrip_kernel, dim3((unsigned)blocks, 2), dim3(256), 0, s, p,
                     (float)((1 << (n_bits - 1)) - 1));
  return hipGetLastError();
}

hipError_t launch_append(const AppendParams& p, hipStream_t s) {
  const int64_t total = (int64_t)p.n_tokens * p.n_kv_heads * (p.row_bytes >> 4);
  if (total <= 0) return hipSuccess;
  if (!p.rope_cos) {
    int log2_vpr = 0;
    while ((16 << log2_vpr) < p.row_bytes) ++log2_vpr;
    if ((16 << log2_vpr) != p.row_bytes || p.n_kv_heads > 32767) return hipErrorInvalidValue;
    const int64_t per_head = (int64_t)p.n_tokens << log2_vpr;
    int64_t bx = (per_head + 255) / 256;
    if (bx > 1024) bx = 1024;
    hipLaunchKernelGGL(append_kernel, dim3((unsigned)bx, (unsigned)(2 * p.n_kv_heads)), dim3(256), 0, s, p, log2_vpr);
    return hipGetLastError();
  }
  int64_t blocks = (total + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (p.elem_is_bf16)
    hipLaunchKernelGGL((append_rope_kernel<__bf16, 8>), dim3((unsigned)blocks, 2), dim3(256), 0, s, p);
  else
    hipLaunchKernelGGL((append_rope_kernel<float, 4>), dim3((unsigned)blocks, 2), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace kvfold
