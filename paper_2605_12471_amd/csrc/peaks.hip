// kvfold_measure_peaks: what the GPU at hand delivers on the two resources the fold step is bound by -- the bf16
// matrix pipes (chunk-prefix attention, paper Sec. 2, is a dense contraction) and HBM reads (a decode-shaped step
// streams the whole cache once).  Two stand-alone kernels; neither is part of the fold step.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "../../include/kvfold.h"
#include "kvfold_host.h"

namespace kvfold {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) unsigned uintx4;

constexpr int kMfmaPerIter = 16;
constexpr double kFlopPerMfma = 2.0 * 32 * 32 * 16;

// One workgroup of four wavefronts per CU (the LDS request keeps a second one out), each wavefront issuing
// independent 32x32x16 bf16 matrix instructions back to back: eight accumulators, so that no instruction waits for
// the result of the one before.  Operand bits differ from lane to lane and register to register (the power a matrix
// pipe draws, and with it the clock the chip sustains, depends on its data).  One store per lane keeps the work alive.
__global__ void __launch_bounds__(256, 1) mfma_only_kernel(float* out, int iters) {
  extern __shared__ unsigned char whole_lds[];
  const int l = threadIdx.x;
  bf16x8 a[4], b[4];
  for (int i = 0; i < 4; ++i)
    for (int e = 0; e < 8; ++e) {
      a[i][e] = (__bf16)(0.0078125f * (float)((l * 7 + i * 3 + e * 5) % 61 - 30));
      b[i][e] = (__bf16)(0.0078125f * (float)((l * 5 + i * 11 + e * 3) % 59 - 29));
    }
  floatx16 acc[8];
  for (int k = 0; k < 8; ++k)
    for (int r = 0; r < 16; ++r) acc[k][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < kMfmaPerIter; ++i)
      asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[i & 7]) : "v"(a[i & 3]), "v"(b[(i >> 2) & 3]));
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");  // the last matrix results are read by ordinary vector adds below
  float sum = 0.f;
  for (int k = 0; k < 8; ++k)
    for (int r = 0; r < 16; ++r) sum += acc[k][r];
  out[(size_t)blockIdx.x * blockDim.x + l] = sum + (float)whole_lds[0] * 0.f;
}

// Grid-stride streaming read, 16 bytes per lane, four loads in flight per lane; one store per lane at the end.
__global__ void __launch_bounds__(256) read_kernel(const uintx4* __restrict__ src, size_t n_vec, unsigned* out) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  unsigned acc = 0;
  for (; i + 3 * stride < n_vec; i += 4 * stride) {
    const uintx4 v0 = __builtin_nontemporal_load(src + i), v1 = __builtin_nontemporal_load(src + i + stride);
    const uintx4 v2 = __builtin_nontemporal_load(src + i + 2 * stride), v3 = __builtin_nontemporal_load(src + i + 3 * stride);
    acc ^= v0.x ^ v0.y ^ v0.z ^ v0.w ^ v1.x ^ v1.y ^ v1.z ^ v1.w ^ v2.x ^ v2.y ^ v2.z ^ v2.w ^ v3.x ^ v3.y ^ v3.z ^ v3.w;
  }
  for (; i < n_vec; i += stride) {
    const uintx4 v = __builtin_nontemporal_load(src + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

struct Buffers {
  void* big = nullptr;
  void* small = nullptr;
  hipEvent_t e0 = nullptr, e1 = nullptr;
  ~Buffers() {
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (big) (void)hipFree(big);
    if (small) (void)hipFree(small);
  }
};

struct DeviceScope {
  int prev = -1;
  hipError_t err;
  explicit DeviceScope(int device) {
    err = hipGetDevice(&prev);
    if (err == hipSuccess && prev != device) err = hipSetDevice(device);
  }
  ~DeviceScope() {
    if (prev >= 0) (void)hipSetDevice(prev);
  }
};

}  // namespace
}  // namespace kvfold

using namespace kvfold;

#define PEAKS_HIP(call)                        \
  do {                                         \
    hipError_t e_ = (call);                    \
    if (e_ != hipSuccess) return hip_fail(e_); \
  } while (0)

extern "C" int kvfold_measure_peaks(int32_t device, double* mfma_bf16_tflops, double* hbm_read_gbps) {
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || device < 0 || device >= n_dev) {
    (void)hipGetLastError();
    return KVFOLD_ERR_INVALID_ARG;
  }
  DeviceScope scope(device);
  if (scope.err != hipSuccess) return hip_fail(scope.err);
  hipDeviceProp_t prop;
  PEAKS_HIP(hipGetDeviceProperties(&prop, device));
  const int n_cu = prop.multiProcessorCount;
  Buffers b;
  PEAKS_HIP(hipEventCreate(&b.e0));
  PEAKS_HIP(hipEventCreate(&b.e1));
  constexpr int kReadBlocksPerCu = 8;
  const size_t small_bytes = (size_t)n_cu * kReadBlocksPerCu * 256 * sizeof(float);
  PEAKS_HIP(hipMalloc(&b.small, small_bytes));

  if (mfma_bf16_tflops) {
    // one resident workgroup per CU: ask for more than half of the CU's LDS
    const int lds_bytes = 96 * 1024;
    PEAKS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(mfma_only_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  lds_bytes));
    const int iters = 200000;  // 3.2 million matrix instructions per wavefront: about 50 ms, long enough for the clock to settle
    double sum_ms = 0.0;
    for (int pass = 0; pass < 4; ++pass) {
      PEAKS_HIP(hipEventRecord(b.e0, nullptr));
      hipLaunchKernelGGL(mfma_only_kernel, dim3(n_cu), dim3(256), lds_bytes, nullptr, static_cast<float*>(b.small), iters);
      PEAKS_HIP(hipGetLastError());
      PEAKS_HIP(hipEventRecord(b.e1, nullptr));
      PEAKS_HIP(hipEventSynchronize(b.e1));
      float ms = 0.f;
      PEAKS_HIP(hipEventElapsedTime(&ms, b.e0, b.e1));
      if (pass > 0) sum_ms += ms;
    }
    *mfma_bf16_tflops = (double)n_cu * 4 * iters * kMfmaPerIter * kFlopPerMfma / (sum_ms / 3 * 1e-3) / 1e12;
  }

  if (hbm_read_gbps) {
    const size_t bytes = (size_t)2 << 30;
    PEAKS_HIP(hipMalloc(&b.big, bytes));
    PEAKS_HIP(hipMemsetAsync(b.big, 0x5a, bytes, nullptr));
    double sum_ms = 0.0;
    for (int pass = 0; pass < 4; ++pass) {
      PEAKS_HIP(hipEventRecord(b.e0, nullptr));
      hipLaunchKernelGGL(read_kernel, dim3(n_cu * kReadBlocksPerCu), dim3(256), 0, nullptr, static_cast<const uintx4*>(b.big),
                         bytes / sizeof(uintx4), static_cast<unsigned*>(b.small));
      PEAKS_HIP(hipGetLastError());
      PEAKS_HIP(hipEventRecord(b.e1, nullptr));
      PEAKS_HIP(hipEventSynchronize(b.e1));
      float ms = 0.f;
      PEAKS_HIP(hipEventElapsedTime(&ms, b.e0, b.e1));
      if (pass > 0) sum_ms += ms;
    }
    *hbm_read_gbps = (double)bytes / (sum_ms / 3 * 1e-3) / 1e9;
  }
  PEAKS_HIP(hipDeviceSynchronize());
  return KVFOLD_OK;
}
