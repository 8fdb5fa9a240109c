/*
 * c_client.c -- a caller of the fold-step library written in plain C: no Python, no PyTorch, device memory from
 * hipMalloc, the default stream.  It folds a sequence of ragged chunks through one layer (Sec. 2: append the chunk,
 * attend to prefix + causal chunk), and writes what it fed in and what came back to raw files, so that a checker can
 * hold the result against an independent implementation.  It also reads the carried cache back through
 * kvfold_cache_view and compares it with the rows it appended, and checks two of the interface's error returns.
 *
 *   kvfold_c_client OUTDIR Hq Hkv d dtype(0 = fp32, 1 = bf16) seed C1 [C2 ...]
 *
 * Files in OUTDIR (element bits as the library sees them, chunks concatenated): q.bin [T][Hq][d], k.bin / v.bin
 * [T][Hkv][d], out.bin [T][Hq][d], lse.bin (per chunk [Hq][C] float), cache_k.bin / cache_v.bin [Hkv][T][d].
 * Inputs are multiples of 1/16 in [-2, 2] from a 64-bit linear congruential generator: exact in bf16 and fp32.
 * Exit status 0 and a last line "ok" on success.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "kvfold.h"

#define HIP_OK(call)                                                                       \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess) {                                                                \
      fprintf(stderr, "%s:%d: %s -> %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
      return 2;                                                                            \
    }                                                                                      \
  } while (0)

#define KV_OK(call)                                                                                     \
  do {                                                                                                  \
    int s_ = (call);                                                                                    \
    if (s_ != KVFOLD_OK) {                                                                              \
      fprintf(stderr, "%s:%d: %s -> %d (%s), hip error %d\n", __FILE__, __LINE__, #call, s_,            \
              kvfold_status_string(s_), kvfold_last_hip_error());                                       \
      return 3;                                                                                         \
    }                                                                                                   \
  } while (0)

static uint64_t g_state;

static float draw(void) { /* k/16, k = -32 .. 32 */
  g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
  return (float)((int)((g_state >> 33) % 65u) - 32) / 16.0f;
}

/* Fill n elements of the mode's type; every drawn value is exact in bf16, whose bits are the float's upper half. */
static void fill(void* dst, size_t n, int bf16) {
  for (size_t i = 0; i < n; ++i) {
    float x = draw();
    if (bf16) {
      uint32_t u;
      memcpy(&u, &x, 4);
      ((uint16_t*)dst)[i] = (uint16_t)(u >> 16);
    } else {
      ((float*)dst)[i] = x;
    }
  }
}

static FILE* open_out(const char* dir, const char* name) {
  char path[4096];
  snprintf(path, sizeof path, "%s/%s", dir, name);
  return fopen(path, "wb");
}

int main(int argc, char** argv) {
  if (argc < 8) {
    fprintf(stderr, "usage: %s OUTDIR Hq Hkv d dtype seed C1 [C2 ...]\n", argv[0]);
    return 1;
  }
  const char* dir = argv[1];
  const int Hq = atoi(argv[2]), Hkv = atoi(argv[3]), d = atoi(argv[4]), bf16 = atoi(argv[5]);
  g_state = strtoull(argv[6], NULL, 10);
  const int n_chunks = argc - 7;
  int64_t total = 0;
  int c_max = 0;
  for (int i = 0; i < n_chunks; ++i) {
    int c = atoi(argv[7 + i]);
    if (c < 1) return 1;
    total += c;
    if (c > c_max) c_max = c;
  }
  const size_t es = bf16 ? 2 : 4;

  HIP_OK(hipSetDevice(0));
  kvfold_config_t cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.struct_size = (uint32_t)sizeof cfg;
  cfg.n_layers = 1;
  cfg.n_q_heads = Hq;
  cfg.n_kv_heads = Hkv;
  cfg.head_dim = d;
  cfg.chunk_tokens = c_max;
  cfg.capacity_tokens = total;
  cfg.dtype = bf16 ? KVFOLD_BF16 : KVFOLD_F32;
  cfg.device = 0;
  /* caller-owned K/V storage: the size the library asks for, allocated here */
  const size_t kv_bytes = kvfold_cache_bytes_required(&cfg);
  if (kv_bytes != (size_t)2 * Hkv * total * d * es) {
    fprintf(stderr, "bytes_required %zu\n", kv_bytes);
    return 4;
  }
  void* kv_buf = NULL;
  HIP_OK(hipMalloc(&kv_buf, kv_bytes));
  cfg.kv_buffer = kv_buf;
  cfg.kv_buffer_bytes = kv_bytes;
  kvfold_cache_t* cache = NULL;
  KV_OK(kvfold_cache_create(&cfg, &cache));

  const size_t q_max = (size_t)c_max * Hq * d, kv_max = (size_t)c_max * Hkv * d;
  void *hq = malloc(q_max * es), *hk = malloc(kv_max * es), *hv = malloc(kv_max * es), *hout = malloc(q_max * es);
  float* hlse = (float*)malloc((size_t)Hq * c_max * 4);
  void* appended_k = malloc((size_t)total * Hkv * d * es);
  void* appended_v = malloc((size_t)total * Hkv * d * es);
  void *dq, *dk, *dv, *dout, *dlse;
  HIP_OK(hipMalloc(&dq, q_max * es));
  HIP_OK(hipMalloc(&dk, kv_max * es));
  HIP_OK(hipMalloc(&dv, kv_max * es));
  HIP_OK(hipMalloc(&dout, q_max * es));
  HIP_OK(hipMalloc(&dlse, (size_t)Hq * c_max * 4));
  FILE *fq = open_out(dir, "q.bin"), *fk = open_out(dir, "k.bin"), *fv = open_out(dir, "v.bin");
  FILE *fo = open_out(dir, "out.bin"), *fl = open_out(dir, "lse.bin");
  if (!hq || !hk || !hv || !hout || !hlse || !appended_k || !appended_v || !fq || !fk || !fv || !fo || !fl) return 5;

  int64_t pos = 0;
  for (int i = 0; i < n_chunks; ++i) {
    const int C = atoi(argv[7 + i]);
    const size_t nq = (size_t)C * Hq * d, nkv = (size_t)C * Hkv * d;
    fill(hq, nq, bf16);
    fill(hk, nkv, bf16);
    fill(hv, nkv, bf16);
    memcpy((char*)appended_k + (size_t)pos * Hkv * d * es, hk, nkv * es);
    memcpy((char*)appended_v + (size_t)pos * Hkv * d * es, hv, nkv * es);
    HIP_OK(hipMemcpy(dq, hq, nq * es, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dk, hk, nkv * es, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(dv, hv, nkv * es, hipMemcpyHostToDevice));
    if (i == 0) { /* a step at the wrong position is refused and changes nothing */
      int s = kvfold_step_ex(cache, 0, dq, dk, dv, C, 1, dout, NULL, NULL);
      if (s != KVFOLD_ERR_POSITION || kvfold_cache_length(cache, 0) != 0) {
        fprintf(stderr, "wrong-position step returned %d\n", s);
        return 6;
      }
    }
    KV_OK(kvfold_step_ex(cache, 0, dq, dk, dv, C, pos, dout, (float*)dlse, NULL));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(hout, dout, nq * es, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(hlse, dlse, (size_t)Hq * C * 4, hipMemcpyDeviceToHost));
    fwrite(hq, es, nq, fq);
    fwrite(hk, es, nkv, fk);
    fwrite(hv, es, nkv, fv);
    fwrite(hout, es, nq, fo);
    fwrite(hlse, 4, (size_t)Hq * C, fl);
    pos += C;
    if (kvfold_cache_length(cache, 0) != pos) return 7;
    printf("chunk %d: %d rows, cache length %lld\n", i, C, (long long)pos);
  }
  fclose(fq), fclose(fk), fclose(fv), fclose(fo), fclose(fl);

  /* the cache is full: one more row is refused */
  if (kvfold_step_ex(cache, 0, dq, dk, dv, 1, pos, dout, NULL, NULL) != KVFOLD_ERR_CAPACITY) return 8;

  /* read the carried state back, head-major, and hold it against the token-major rows that were appended */
  void *k_dev = NULL, *v_dev = NULL;
  int64_t row_stride = 0, head_stride = 0;
  KV_OK(kvfold_cache_view(cache, 0, &k_dev, &v_dev, &row_stride, &head_stride));
  if ((char*)k_dev != (char*)kv_buf || row_stride != d || head_stride != total * d) return 9;
  void* back = malloc((size_t)total * d * es);
  FILE *fck = open_out(dir, "cache_k.bin"), *fcv = open_out(dir, "cache_v.bin");
  if (!back || !fck || !fcv) return 5;
  for (int which = 0; which < 2; ++which) {
    for (int h = 0; h < Hkv; ++h) {
      const char* src = (const char*)(which ? v_dev : k_dev) + (size_t)h * head_stride * es;
      HIP_OK(hipMemcpy(back, src, (size_t)total * d * es, hipMemcpyDeviceToHost));
      fwrite(back, es, (size_t)total * d, which ? fcv : fck);
      const char* fed = (const char*)(which ? appended_v : appended_k);
      for (int64_t r = 0; r < total; ++r)
        if (memcmp((char*)back + (size_t)r * d * es, fed + ((size_t)r * Hkv + h) * d * es, (size_t)d * es) != 0) {
          fprintf(stderr, "cache %s head %d row %lld differs from the appended row\n", which ? "V" : "K", h, (long long)r);
          return 10;
        }
    }
  }
  fclose(fck), fclose(fcv);

  KV_OK(kvfold_cache_destroy(cache));
  HIP_OK(hipFree(kv_buf)); /* caller-owned storage outlives the cache */
  HIP_OK(hipFree(dq));
  HIP_OK(hipFree(dk));
  HIP_OK(hipFree(dv));
  HIP_OK(hipFree(dout));
  HIP_OK(hipFree(dlse));
  free(hq), free(hk), free(hv), free(hout), free(hlse), free(appended_k), free(appended_v), free(back);
  printf("ok\n");
  return 0;
}
