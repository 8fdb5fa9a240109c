/*
 * kvfold.h -- C ABI of the KV-Fold fold step for one AMD MI355X (gfx950).
 *
 * The fold step is the per-layer attention-with-carried-cache operation of the
 * paper's Sec. 2 ("KV-Fold"): when chunk t is processed, the queries of its C
 * new tokens attend to keys K_{0:t} = [K_0; ...; K_t] and values V_{0:t} --
 * every earlier chunk in full plus a causal mask inside the chunk -- and the
 * chunk's own K/V rows are appended to the cache that is carried to chunk t+1
 * (Fig. 2; the recurrence (K^(t),V^(t)) = F((K^(t-1),V^(t-1)), x_t) and its
 * left-fold form in "A recurrent view").  Position ids continue from tC
 * (Sec. 2), which this interface expresses as `pos_offset`.
 *
 * All entry points are plain C, return an `int` status (0 = KVFOLD_OK,
 * negative = error), never throw, never print and never abort.  Every error
 * except KVFOLD_ERR_HIP is found before anything is enqueued: nothing has run
 * and the cache is unchanged.  KVFOLD_ERR_HIP from a step means the HIP runtime
 * refused a launch (everything a valid configuration could be refused for is
 * settled by kvfold_cache_create): the layer's length is unchanged, but
 * kernels of that step launched before the failure stay enqueued and rows
 * [length, length + n_tokens) of the layer may have been written.
 *
 * Pointer kinds are stated per argument: "host" pointers are ordinary process
 * memory, "device" pointers are HIP device allocations on the cache's device.
 */
#ifndef KVFOLD_H
#define KVFOLD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kvfold_cache kvfold_cache_t; /* opaque; created/destroyed by the library */

typedef enum { KVFOLD_F32 = 0, KVFOLD_BF16 = 1 } kvfold_dtype_t;

enum {
  KVFOLD_OK = 0,
  KVFOLD_ERR_INVALID_ARG = -1, /* null pointer, non-positive size, bad struct_size          */
  KVFOLD_ERR_BAD_LAYER = -2,   /* layer outside [0, n_layers)                                */
  KVFOLD_ERR_POSITION = -3,    /* pos_offset != current length of that layer's cache         */
  KVFOLD_ERR_CAPACITY = -4,    /* length + n_tokens > capacity_tokens (cache untouched)      */
  KVFOLD_ERR_UNSUPPORTED = -5, /* head_dim not in {64,128}, Hq % Hkv != 0, unknown dtype ... */
  KVFOLD_ERR_OOM = -6,         /* device allocation failed / caller buffer too small         */
  KVFOLD_ERR_HIP = -7,         /* any other HIP runtime error (see kvfold_last_hip_error)    */
  KVFOLD_ERR_SCRATCH = -8      /* kvfold_step_noalloc: the step exceeds the static scratch   */
};

/*
 * Configuration of a cache.  Shapes follow the paper's models (Tab. 4 caption:
 * Llama-3.1-8B has 32 layers x 8 KV heads x 128 dims, K and V, 2 bytes in
 * bf16 = 131,072 bytes per token).  Grouped-query heads: query head h reads KV
 * head h / (n_q_heads / n_kv_heads).
 */
typedef struct {
  uint32_t struct_size;    /* must be sizeof(kvfold_config_t)                                 */
  int32_t n_layers;        /* independent per-layer caches, >= 1                              */
  int32_t n_q_heads;       /* Hq, multiple of n_kv_heads                                      */
  int32_t n_kv_heads;      /* Hkv, 1 .. 32767                                                 */
  int32_t head_dim;        /* d: 64 or 128                                                    */
  int32_t chunk_tokens;    /* C used by kvfold_step(); also the largest n_tokens of _ex; >= 1 */
  int64_t capacity_tokens; /* rows reserved per layer; the cache grows in place up to this    */
  int32_t dtype;           /* kvfold_dtype_t: element type of q, k_new, v_new, cache and out  */
  float softmax_scale;     /* logits are scaled by this; 0 selects 1/sqrt(head_dim)           */
  int32_t device;          /* HIP device ordinal the cache lives on                           */
  void* kv_buffer;         /* device; optional caller-owned storage for the K/V rows, at      */
                           /* least kvfold_cache_bytes_required() bytes, 256-byte aligned;    */
                           /* NULL = the library allocates (and frees) it                     */
  size_t kv_buffer_bytes;  /* size of kv_buffer when it is given                              */
} kvfold_config_t;

/*
 * Bytes of K/V storage a cache of this configuration needs:
 * n_layers * 2 * n_kv_heads * capacity_tokens * head_dim * elem_size (the
 * paper's per-token figure times capacity; Tab. 4).  Host-only, touches no
 * GPU.  Returns 0 for an invalid configuration.
 */
size_t kvfold_cache_bytes_required(const kvfold_config_t* cfg /* host */);

/*
 * Create an empty cache (the fold's initial accumulator (empty, empty), Sec. 2).
 * Layout in HBM: K rows [layer][kv_head][capacity][head_dim], then V rows with
 * the same shape; a row never moves once written.  Also reserves a fixed
 * workspace for split-prefix partial results so that steps allocate nothing.
 * cfg: host.  out_cache: host, receives the handle (NULL on error).
 */
int kvfold_cache_create(const kvfold_config_t* cfg, kvfold_cache_t** out_cache);

/*
 * One fold step on one layer (Sec. 2): append the chunk's C = cfg.chunk_tokens
 * new K/V rows at rows [pos_offset, pos_offset + C) of the layer's cache, then
 * compute out[i][h] = softmax_j(scale * q[i][h] . K[h/G][j]) V[h/G][j] over the
 * keys j <= pos_offset + i.
 *
 *   q      device, [C][Hq][d]   queries, used as given (already position-rotated)
 *   k_new  device, [C][Hkv][d]  new key rows, token-major
 *   v_new  device, [C][Hkv][d]  new value rows
 *   pos_offset  absolute position of the chunk's first token; must equal the
 *               layer's current length (else KVFOLD_ERR_POSITION)
 *   out    device, [C][Hq][d]   attention output, element type = cfg.dtype
 *   stream hipStream_t (NULL = default stream)
 *
 * Asynchronous: work is enqueued on `stream`, nothing is synchronised or
 * allocated.  The caller keeps q/k_new/v_new/out alive until the stream has
 * passed the step.  Steps on the same cache must be issued from one host
 * thread at a time and be stream-ordered (same stream or explicit events):
 * the split workspace is shared by all layers of a cache.  The host-side
 * length of the layer advances by C when the call returns KVFOLD_OK.
 */
int kvfold_step(kvfold_cache_t* cache, int layer, const void* q, const void* k_new, const void* v_new,
                int64_t pos_offset, void* out, void* stream);

/*
 * Same step with a ragged chunk (1 <= n_tokens <= cfg.chunk_tokens; the paper's
 * question chunk after the data chunks has its own length, Sec. 4) and an
 * optional log-sum-exp output:
 *   lse  device or NULL, [Hq][n_tokens] float: natural-log sum of exp(scaled
 *        logits) over the visible keys of each row (lets a caller recover the
 *        softmax weight of any single key).
 */
int kvfold_step_ex(kvfold_cache_t* cache, int layer, const void* q, const void* k_new, const void* v_new,
                   int32_t n_tokens, int64_t pos_offset, void* out, float* lse, void* stream);

/*
 * Same step for callers that hold q and k_new UNROTATED: the rotary position
 * embedding of the new tokens at their absolute positions pos_offset + i is
 * applied inside the step (Sec. 2: the position ids of chunk t go on from the
 * absolute position tC, which keeps the rotations aligned with the unchunked
 * sequence) -- to the K rows as they are appended (the cache holds rotated
 * keys, as a model's cache does) and to the queries as the attention kernel
 * loads them; V is untouched.
 *   rope_cos, rope_sin  device, [n_tokens][head_dim/2] float, 16-byte aligned:
 *        cosine and sine of the angle of pair j at row i's absolute position
 *        (what a model's rotary cache holds for positions pos_offset ..
 *        pos_offset + n_tokens - 1; frequencies and any scaling are the
 *        caller's).  Both required, else KVFOLD_ERR_INVALID_ARG.
 * Pairing is the half-split layout of the Llama family: element j rotates with
 * element j + head_dim/2,
 *        x'_j = x_j cos_j - x_{j+d/2} sin_j,  x'_{j+d/2} = x_{j+d/2} cos_j + x_j sin_j,
 * in fp32 (the product with the sine rounded first, then one fused multiply-
 * add) and rounded to the mode's element type.  The result is bit for bit
 * what kvfold_step_ex returns, and leaves in the cache, for inputs rotated that
 * way beforehand.  All other arguments, layouts and errors as kvfold_step_ex.
 */
int kvfold_step_rope(kvfold_cache_t* cache, int layer, const void* q, const void* k_new, const void* v_new,
                     int32_t n_tokens, int64_t pos_offset, const float* rope_cos, const float* rope_sin, void* out,
                     float* lse, void* stream);

/*
 * The same step under the mask of the streaming baseline the paper compares with (Sec. 6, "Comparison to
 * StreamingLLM": a few attention-sink tokens kept from the start of the sequence plus a sliding window of
 * recent tokens, 4 + 1020 in its experiments, evicted keys losing their place but kept ones keeping their
 * original positions).  The chunk's rows are appended exactly as in kvfold_step_ex (the cache stays complete,
 * so plain and windowed steps can be mixed on one cache), but the row at absolute position p = pos_offset + i
 * attends only to the keys
 *        j < n_sink   or   p - window < j <= p
 * (its own key is one of the `window` recent ones).  n_sink >= 0, 1 <= window <= 2^30, else
 * KVFOLD_ERR_INVALID_ARG; a window that covers the whole cache gives the result of kvfold_step_ex.  Work and
 * HBM reads are proportional to n_sink + window, not to the cache length: key tiles between the sinks and the
 * window are never touched.  All other arguments, layouts and errors as kvfold_step_ex.
 */
int kvfold_step_window(kvfold_cache_t* cache, int layer, const void* q, const void* k_new, const void* v_new,
                       int32_t n_tokens, int64_t pos_offset, int32_t n_sink, int64_t window, void* out, float* lse,
                       void* stream);

/*
 * kvfold_step_ex for callers that can neither allocate device memory nor tolerate a library that does: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, layouts,
 * results and errors as kvfold_step_ex, but the partial results of a split key range go to a fixed array that
 * is part of the library's code object (65 MiB per GPU, held until the process ends) instead of the cache's
 * workspace; the call allocates nothing and frees nothing.  Limit: n_tokens * n_q_heads <= 65536 (two pieces of
 * the step must fit the array's 131072 (row, piece) slots), else KVFOLD_ERR_SCRATCH and nothing is enqueued;
 * the number of pieces the planner may use is bounded by the same array.  Every call on one GPU shares that
 * GPU's array: calls whose work overlaps in time on one GPU (different streams, different caches) race on it;
 * stream-ordered calls are safe, and nothing in the array has to be cleared between calls (every slot a merge
 * reads was written by the attention kernel just before it).
 */
int kvfold_step_noalloc(kvfold_cache_t* cache, int layer, const void* q, const void* k_new, const void* v_new,
                        int32_t n_tokens, int64_t pos_offset, void* out, float* lse, void* stream);

/*
 * Destroy a cache: synchronises the device, frees library-owned memory (never
 * a caller-provided kv_buffer).  NULL is a no-op returning KVFOLD_OK.
 */
int kvfold_cache_destroy(kvfold_cache_t* cache);

/* Current number of rows held for `layer`; negative status on error. Host-only. */
int64_t kvfold_cache_length(const kvfold_cache_t* cache, int layer);

/*
 * Device pointers to the first K and V row of `layer` (KV head 0) and the
 * strides, in elements, between consecutive rows and consecutive KV heads.
 * Any output pointer may be NULL.  The rows are the complete recurrent state
 * (Sec. 2, "A recurrent view"): copying rows [0, length) out and back restores
 * a fold.  Host-only.
 */
int kvfold_cache_view(const kvfold_cache_t* cache, int layer, void** k_dev, void** v_dev,
                      int64_t* row_stride_elems, int64_t* head_stride_elems);

/*
 * Rewind `layer` (-1 = every layer) to `new_len` rows, 0 = reset.  Shrink only:
 * new_len must not exceed the current length of the layer (of any layer when
 * layer is -1), else KVFOLD_ERR_POSITION and nothing changes.  Rows stay in HBM;
 * the cache accumulates and never overwrites (Sec. 3), so re-running the
 * steps after a rewind re-appends identical rows.  Host-only; the caller orders
 * it against in-flight steps.
 */
int kvfold_cache_truncate(kvfold_cache_t* cache, int layer, int64_t new_len);

/*
 * Set the host-side length of `layer` (-1 = every layer) to `new_len`.
 * new_len <= capacity; rows are left as they are in HBM.  Shrinking rewinds a
 * fold (re-running a step re-appends identical rows); growing adopts rows a
 * caller has copied in through kvfold_cache_view (resume).  Host-only; the
 * caller orders it against in-flight steps.
 */
int kvfold_cache_set_length(kvfold_cache_t* cache, int layer, int64_t new_len);

/*
 * Storage perturbation of the carried cache (Sec. 8, Discussion: a per-step
 * quantisation round trip bf16 -> intN -> bf16).  n_bits = 8 or 4: from now on
 * every step passes the K and V rows it appends through that integer width and
 * back, in place, before its queries attend to them; 0 switches it off.  The
 * paper names no quantiser; the one used: a group is the head_dim elements of
 * one (token, KV head) row, symmetric, scale = max|x| / (2^(N-1) - 1), code =
 * round-half-even(x / scale) clamped to +-(2^(N-1) - 1), x' = code * scale, in
 * fp32, stored as bf16 (RNE); an all-zero row stays zero.  bf16 caches only
 * (KVFOLD_ERR_UNSUPPORTED otherwise); other values KVFOLD_ERR_INVALID_ARG.
 * Host-only; applies to steps enqueued after the call.
 */
int kvfold_cache_set_storage_roundtrip(kvfold_cache_t* cache, int32_t n_bits);

/*
 * Tuning knobs for measurements (defaults are chosen automatically per step).
 *   KVFOLD_TUNE_SPLITS         number of prefix splits of the attention kernel; 0 = automatic.
 *                              Clamped to what the split workspace and the key range allow.
 *   KVFOLD_TUNE_UNITS_PER_WAVE 32-row query blocks owned by one wavefront of the bf16 kernel:
 *                              1 or 2; 0 = automatic.
 *   KVFOLD_TUNE_PAIR_UNITS     two-unit kernel: each wavefront owns an early and a late row
 *                              block of the chunk (evens out the causal part); 0 = automatic (single
 *                              round of workgroups), 1 = never, 2 = always.
 *   KVFOLD_TUNE_FUSED_APPEND   bf16 mode: the attention kernel copies the chunk's rows into the cache itself
 *                              (and reads the chunk's own rows from k_new / v_new) whenever neither rotary
 *                              embedding nor a storage round trip is in play and n_tokens * n_kv_heads * head_dim * 2 bytes is
 *                              below 2^32 (the kernel addresses the chunk with 32-bit byte offsets; larger
 *                              chunks go through the separate append kernel); 0 = automatic, 1 = never.
 *                              Either way k_new / v_new must stay valid until the step's work on the
 *                              stream is done, and the cache ends up with the same bits.
 * Returns KVFOLD_ERR_INVALID_ARG for an unknown knob or a value out of range.  Host-only.
 */
enum { KVFOLD_TUNE_SPLITS = 0, KVFOLD_TUNE_UNITS_PER_WAVE = 1, KVFOLD_TUNE_PAIR_UNITS = 2, KVFOLD_TUNE_FUSED_APPEND = 3 };
int kvfold_cache_set_tuning(kvfold_cache_t* cache, int32_t knob, int32_t value);

/*
 * Launch geometry the next step would use for n_tokens rows at length
 * `len_after` (for reports): number of workgroups and prefix splits.
 */
int kvfold_cache_plan(const kvfold_cache_t* cache, int32_t n_tokens, int64_t len_after, int32_t* n_workgroups,
                      int32_t* n_splits);

/*
 * The same launch geometry without a cache or a device: what a cache created from `cfg` on a GPU with
 * `n_compute_units` CUs would use for a step of n_tokens rows that leaves the cache at `len_after` rows, with
 * every tuning knob at automatic; window > 0 asks for the sink + sliding-window step (kvfold_step_window),
 * window = 0 for the plain one.  Host-only, touches no GPU.  KVFOLD_ERR_INVALID_ARG / _UNSUPPORTED as for
 * create, and for n_tokens, len_after, n_sink or window outside the configuration, or out == NULL.
 */
typedef struct {
  int32_t n_workgroups;    /* workgroups of the attention kernel                                        */
  int32_t n_splits;        /* pieces the key range is cut into (> 1: a merge kernel follows)            */
  int32_t units_per_wave;  /* 32-row query blocks per wavefront (bf16: 1 or 2; fp32: 1)                 */
  int32_t tiles_per_split; /* 64-key tiles per piece                                                    */
  int32_t fused_append;    /* 1: the attention kernel appends the chunk's rows itself (kvfold_step_ex)  */
  int32_t pair_units;      /* 1: every wavefront owns an early and a late row block of the chunk        */
  int32_t pair_order;      /* 1: workgroups ordered so that each CU gets a heavy and a light one        */
} kvfold_plan_t;
int kvfold_plan_for(const kvfold_config_t* cfg /* host */, int32_t n_compute_units, int32_t n_tokens, int64_t len_after,
                    int32_t n_sink, int64_t window, kvfold_plan_t* out /* host */);

/*
 * Per-kernel timing for measurements.  Between _begin and _end every step additionally records
 * HIP events on the step's stream around each of its kernels (append, attention, merge), at most
 * `max_steps` steps (further steps run untimed).  _end synchronises the device, adds up the
 * elapsed times in milliseconds, releases the events and returns to normal operation.  A step
 * whose attention kernel appended by itself counts wholly as attention time.  Any
 * output pointer may be NULL.  Event creation makes _begin the only call besides create/destroy
 * that allocates.
 */
int kvfold_cache_profile_begin(kvfold_cache_t* cache, int32_t max_steps);
int kvfold_cache_profile_end(kvfold_cache_t* cache, int32_t* n_steps /* host */, double* append_ms /* host */,
                             double* attention_ms /* host */, double* merge_ms /* host */);

/*
 * What this GPU delivers, for reports that quote an achieved rate beside the datasheet's (not part of the fold
 * step): two stand-alone kernels, timed with HIP events on the default stream of `device`.
 *   mfma_bf16_tflops  host or NULL: rate of a loop of nothing but 32x32x16 bf16 matrix instructions, one wavefront
 *                     on every SIMD of every CU, operands in registers, no memory traffic -- the ceiling of any
 *                     bf16 contraction on this part at the clock it sustains under that load.
 *   hbm_read_gbps     host or NULL: rate of a plain streaming read (16 bytes per lane) of a 2 GiB buffer, far beyond
 *                     every cache -- the ceiling of a read-bound step such as a decode-shaped one.
 * Each figure is the mean of three timed passes after a warm-up pass (the matrix passes take about 50 ms each, so
 * that the clock settles under the load).  Allocates (and frees) the 2 GiB buffer and a small output buffer,
 * synchronises the device; takes about 0.25 s.  KVFOLD_ERR_INVALID_ARG for a bad device ordinal,
 * KVFOLD_ERR_OOM / KVFOLD_ERR_HIP from the runtime.
 */
int kvfold_measure_peaks(int32_t device, double* mfma_bf16_tflops, double* hbm_read_gbps);

/* Static, human-readable name of a status code. */
const char* kvfold_status_string(int status);

/* hipError_t value of the last HIP failure seen by this thread's calls (0 = none). */
int kvfold_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* KVFOLD_H */
