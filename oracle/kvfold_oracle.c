/*
 * kvfold_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * Plain fp64 CPU reference for the KV-Fold fold step (paper Sec. 2, "KV-Fold":
 * at chunk t the queries of the new tokens attend to the keys/values
 * K_{0:t} = [K_0; ...; K_t], V_{0:t}; the chunk's own K/V rows are appended
 * to the carried cache, earlier rows are never touched -- Fig. 2, and the
 * recurrence (K^(t),V^(t)) = F((K^(t-1),V^(t-1)), x_t) of "A recurrent view").
 *
 * The method is a reorganisation of ordinary causal attention (Sec. 5 says
 * so itself: it saves neither memory nor FLOPs in total), so the oracle is the plain
 * definition written out: one dot product per (query row, key), a two-pass
 * softmax over the visible keys, a weighted sum of value rows.  No tiling,
 * no online softmax, no fusion.  Everything is double precision.
 *
 * This file shares nothing with the HIP library (no headers, no helpers).
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may
 * load it.
 *
 * Layouts (all C-contiguous, double):
 *   q      [C][Hq][d]        queries of the chunk, token-major
 *   k_new  [C][Hkv][d]       new key rows, token-major (same for v_new)
 *   Kc,Vc  [Hkv][cap][d]     carried cache, head-major; rows [0,len) valid
 *   out    [nrows][Hq][d]    one slab per requested row
 *   lse    [nrows][Hq]       log-sum-exp of the scaled logits (natural log)
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Cache carry (Fig. 2: the prefix is passed on "as is", the new rows are
 * appended): rows [len, len+C) of every KV head receive the chunk's rows.
 * Works on raw element bytes so that it also defines the bit pattern the
 * device cache must hold. elem_bytes is the size of one element. */
int kvfold_oracle_append_bytes(unsigned char *cache, int64_t Hkv, int64_t cap,
                               int64_t d, int64_t len,
                               const unsigned char *rows_new, int64_t C,
                               int64_t elem_bytes)
{
    if (len < 0 || C < 0 || len + C > cap) return -1;
    const size_t row = (size_t)d * (size_t)elem_bytes;
    for (int64_t i = 0; i < C; ++i)
        for (int64_t g = 0; g < Hkv; ++g)
            memcpy(cache + ((size_t)g * (size_t)cap + (size_t)(len + i)) * row,
                   rows_new + ((size_t)i * (size_t)Hkv + (size_t)g) * row, row);
    return 0;
}

/* Chunk-prefix attention for a list of chunk rows (Sec. 2: queries Q_t of the
 * new tokens, keys K_{0:t}; positions continue from tC, so chunk row i sits at
 * absolute position len_prev+i and, causally, sees keys 0..len_prev+i).
 *
 *   rows[r]   chunk-relative row index in [0,C)
 *   len_prev  cache length BEFORE this chunk was appended; the cache passed in
 *             must already contain the chunk's own rows at [len_prev,len_prev+C)
 *   Query head h reads KV head h / (Hq/Hkv) (contiguous groups).
 *   weights   optional [nrows][Hq][len_prev+C]: softmax weight of every key
 *             (0 for invisible keys); NULL to skip.
 */
int kvfold_oracle_attend_rows(const double *Kc, const double *Vc, int64_t Hkv,
                              int64_t cap, int64_t d, const double *q,
                              int64_t C, int64_t Hq, int64_t len_prev,
                              double scale, const int64_t *rows, int64_t nrows,
                              double *out, double *lse, double *weights)
{
    if (Hq % Hkv != 0 || len_prev < 0 || len_prev + C > cap) return -1;
    for (int64_t r = 0; r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= C) return -2;
    const int64_t G = Hq / Hkv;
    const int64_t Ltot = len_prev + C;
    int fail = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t r = 0; r < nrows; ++r) {
        for (int64_t h = 0; h < Hq; ++h) {
            const int64_t i = rows[r];
            const int64_t g = h / G;
            const int64_t n = len_prev + i + 1; /* visible keys 0..n-1 */
            const double *qv = q + ((size_t)i * Hq + h) * d;
            const double *Kg = Kc + (size_t)g * cap * d;
            const double *Vg = Vc + (size_t)g * cap * d;
            double *s = (double *)malloc((size_t)n * sizeof(double));
            if (!s) { fail = 1; continue; }

            /* logits and their maximum */
            double m = -INFINITY;
            for (int64_t j = 0; j < n; ++j) {
                double acc = 0.0;
                for (int64_t x = 0; x < d; ++x) acc += qv[x] * Kg[(size_t)j * d + x];
                s[j] = acc * scale;
                if (s[j] > m) m = s[j];
            }
            /* normaliser */
            double l = 0.0;
            for (int64_t j = 0; j < n; ++j) { s[j] = exp(s[j] - m); l += s[j]; }
            /* weighted sum of values */
            double *o = out + ((size_t)r * Hq + h) * d;
            for (int64_t x = 0; x < d; ++x) o[x] = 0.0;
            for (int64_t j = 0; j < n; ++j) {
                const double p = s[j] / l;
                for (int64_t x = 0; x < d; ++x) o[x] += p * Vg[(size_t)j * d + x];
            }
            if (lse) lse[(size_t)r * Hq + h] = m + log(l);
            if (weights) {
                double *w = weights + ((size_t)r * Hq + h) * Ltot;
                for (int64_t j = 0; j < Ltot; ++j) w[j] = (j < n) ? s[j] / l : 0.0;
            }
            free(s);
        }
    }
    return fail ? -3 : 0;
}

/*
 * The same attention under the mask of the streaming baseline that the paper compares with (Sec. 6,
 * "Comparison to StreamingLLM": a small number of attention-sink tokens kept from the start of the
 * sequence plus a sliding window of recent tokens -- 4 sinks + 1020 recent tokens in its experiments --
 * with position-preserving eviction, i.e. every kept key stays at its original position and nothing is
 * re-anchored).  Reading taken (the paper gives the cache policy, not a per-row rule): the chunk row at
 * absolute position p = len_prev + i attends to key j iff
 *        j <= p   and   ( j < n_sink   or   j > p - window ),
 * so its own key counts as one of the `window` recent tokens, and a row early enough to see everything
 * (p < n_sink + window) is an ordinary causal row.  Keys outside the set get weight exactly 0.
 * Arguments as kvfold_oracle_attend_rows, plus n_sink >= 0 and window >= 1.
 */
int kvfold_oracle_attend_rows_window(const double *Kc, const double *Vc, int64_t Hkv,
                                     int64_t cap, int64_t d, const double *q,
                                     int64_t C, int64_t Hq, int64_t len_prev,
                                     double scale, int64_t n_sink, int64_t window,
                                     const int64_t *rows, int64_t nrows,
                                     double *out, double *lse, double *weights)
{
    if (Hq % Hkv != 0 || len_prev < 0 || len_prev + C > cap) return -1;
    if (n_sink < 0 || window < 1) return -4;
    for (int64_t r = 0; r < nrows; ++r)
        if (rows[r] < 0 || rows[r] >= C) return -2;
    const int64_t G = Hq / Hkv;
    const int64_t Ltot = len_prev + C;
    int fail = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int64_t r = 0; r < nrows; ++r) {
        for (int64_t h = 0; h < Hq; ++h) {
            const int64_t i = rows[r];
            const int64_t g = h / G;
            const int64_t p = len_prev + i; /* absolute position of the row */
            const double *qv = q + ((size_t)i * Hq + h) * d;
            const double *Kg = Kc + (size_t)g * cap * d;
            const double *Vg = Vc + (size_t)g * cap * d;
            double *s = (double *)malloc((size_t)(p + 1) * sizeof(double));
            if (!s) { fail = 1; continue; }

            /* logits of the visible keys and their maximum (the row's own key is always visible) */
            double m = -INFINITY;
            for (int64_t j = 0; j <= p; ++j) {
                const int seen = (j < n_sink) || (j > p - window);
                if (!seen) { s[j] = -INFINITY; continue; }
                double acc = 0.0;
                for (int64_t x = 0; x < d; ++x) acc += qv[x] * Kg[(size_t)j * d + x];
                s[j] = acc * scale;
                if (s[j] > m) m = s[j];
            }
            double l = 0.0;
            for (int64_t j = 0; j <= p; ++j) { s[j] = exp(s[j] - m); l += s[j]; } /* exp(-inf) = 0 */
            double *o = out + ((size_t)r * Hq + h) * d;
            for (int64_t x = 0; x < d; ++x) o[x] = 0.0;
            for (int64_t j = 0; j <= p; ++j) {
                if (s[j] == 0.0) continue;
                const double w = s[j] / l;
                for (int64_t x = 0; x < d; ++x) o[x] += w * Vg[(size_t)j * d + x];
            }
            if (lse) lse[(size_t)r * Hq + h] = m + log(l);
            if (weights) {
                double *w = weights + ((size_t)r * Hq + h) * Ltot;
                for (int64_t j = 0; j < Ltot; ++j) w[j] = (j <= p) ? s[j] / l : 0.0;
            }
            free(s);
        }
    }
    return fail ? -3 : 0;
}

/*
 * Rotary position embedding of the new tokens at their absolute positions (Sec. 2, "KV-Fold":
 * position identifiers of chunk t continue from tC, so the rotations are aligned with the original
 * sequence).  x: [rows][heads][d] fp32, row i belongs to position pos_offset + i; the caller passes
 * the angles of exactly those positions, cos/sin: [rows][d/2] fp32 (a model's rotary cache).
 * Pairing (the paper is silent; the reading taken is the half-split layout of the Llama family):
 * element j pairs with element j + d/2,
 *     out_j       = x_j cos_j - x_{j+d/2} sin_j
 *     out_{j+d/2} = x_{j+d/2} cos_j + x_j sin_j.
 * Precision: the product layer rotates in fp32 and stores the mode dtype, so this is the one place
 * where the oracle works in fp32 too, with the rounding points fixed: the subtrahend / addend
 * product is rounded to fp32, then one fused multiply-add.
 */
int kvfold_oracle_rope_f32(const float *x, int64_t rows, int64_t heads, int64_t d,
                           const float *cosv, const float *sinv, float *out)
{
    if (d % 2) return -1;
    const int64_t hd = d / 2;
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t h = 0; h < heads; ++h) {
            const float *xi = x + ((size_t)i * heads + h) * d;
            float *oi = out + ((size_t)i * heads + h) * d;
            for (int64_t j = 0; j < hd; ++j) {
                const float c = cosv[(size_t)i * hd + j], s = sinv[(size_t)i * hd + j];
                const float lo = xi[j], hi = xi[j + hd];
                const float t0 = hi * s;      /* rounded to fp32 */
                const float t1 = lo * s;
                oi[j] = fmaf(lo, c, -t0);
                oi[j + hd] = fmaf(hi, c, t1);
            }
        }
    return 0;
}

int kvfold_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
