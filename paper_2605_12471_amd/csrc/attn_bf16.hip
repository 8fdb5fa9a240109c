// Chunk-prefix attention of the fold step, bf16 operands on the gfx950 matrix cores.
//
// What it computes (paper Sec. 2, "KV-Fold"): row i of the chunk, query head h, attends to cache
// rows j <= len_prev + i of KV head h / G -- the whole prefix plus the causal part of the chunk
// itself:
//     out[i][h] = sum_j softmax_j(scale * q[i][h] . K[j]) V[j].
// The chunk's rows are either in the cache already (the append kernel ran first) or are read from
// k_new / v_new as handed in while this kernel also copies them into the cache (fused append; a key
// tile with rows on both sides of the old cache's end is filled from both).  Under the sink +
// sliding-window mask (Sec. 6, the streaming baseline) a row sees of those keys only the first
// n_sink and the last `window`, and the key tiles in between are never touched.
//
// Mapping to the machine
//  * Work unit = (32 consecutive chunk rows, one query head).  A wavefront owns QB units, a
//    workgroup 4 wavefronts; all units of a workgroup share one KV head, so a K/V tile staged in
//    LDS is reused across the grouped-query heads, and with QB = 2 every K/V fragment read from
//    LDS feeds two MFMAs.  Units are ordered token-block-major, head-minor, so the wavefronts of a
//    workgroup see (almost) the same key range and only the last tiles need the causal mask.
//  * 64-key K/V tiles travel HBM/L2 -> LDS with global_load_lds_dwordx4 (no registers), several
//    tiles ahead, into rings of NV+1 (K) and NV (V) slots; the XOR swizzle that makes the later
//    LDS reads conflict-free is applied by choosing which 16-byte chunk each lane fetches.
//  * Per tile a wavefront forms S^T = K Q^T with v_mfma_f32_32x32x16_bf16 (keys are the M rows),
//    so each lane ends up with 32 logits of ONE query: row max / row sum are in-lane plus one
//    exchange between lanes l and l^32.  The accumulator layout of S^T is, up to a fixed
//    permutation of the keys inside a 16-key slab, the B-operand layout of the next product
//    O^T = V^T P^T; V^T fragments are read from the row-major V tile with the LDS transpose read
//    (ds_read_b64_tr_b16) using the same permutation, so P never leaves registers.
//  * Software pipeline inside the wavefront, in half tiles of 32 keys: while the matrix pipe forms
//    S^T of half h+1 and then accumulates O^T of half h, the vector ALU turns S^T of half h into P
//    (exp2, bf16 pack, row sums) -- one exp2 behind every MFMA, the first quarter of a half already
//    in the tail of the step before, because a single wavefront hides only about 16-20 cycles of
//    other instructions under each 32-cycle MFMA.
//  * Online softmax in base 2 with ONE vector instruction per logit: the queries are multiplied by
//    scale*log2(e) once (and rounded to bf16 again), and the S^T accumulators start from -m (the
//    running row max) instead of 0, so the matrix pipe delivers S*scale*log2e - m and P is a bare
//    exp2.  m only has to be a reference close enough to the true row max for P to stay inside the
//    float range, so on tiles below the causal horizon no row max is taken at all: the row sum of a
//    half, which is needed anyway, bounds its largest P, and when it passes 2^20 the reference moves
//    up by a whole power of two (O, l and the in-flight logits are corrected exactly).  A row sum
//    beyond 2^60, infinite or NaN means the logits jumped by more than that inside one half; the
//    workgroup then starts over in a mode that takes the exact row max of every half before its
//    exp2 (the mode the masked tiles at the causal horizon always use, stale by at most 2^16).
//    P is rounded to bf16 by the hardware pack convert; row sums add the unrounded fp32 values.
//  * Optional split of the key range over workgroups: partial (max, sum, O) go to a workspace
//    and are merged by the combine kernel.
//  * Start and end of a workgroup are kept short (they are 4 % of a short-prefix launch): the ring is
//    filled before the Q rows are fetched, all Q loads are in flight together, the first reference is
//    set without touching the still-zero O, and the finished O^T is turned in the dead ring space so
//    that every store instruction writes whole rows.
#include <type_traits>

#include "kvfold_internal.h"

namespace kvfold {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(4))) short short4_;
typedef __attribute__((ext_vector_type(8))) short short8_;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) unsigned uintx4;
typedef __attribute__((ext_vector_type(4))) float floatx4;

#define LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(uintptr_t)(p))

__device__ __forceinline__ float pair_max(float x) {
  // lanes l and l^32 exchange x; both end with the maximum
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// One wavefront-wide 1 KiB copy global -> LDS: lane l's 16 bytes, read from base + off, land at
// lds_base + 16*l.  The compiler is not told about the LDS write; ordering is done by hand with
// wait_vm<> + barrier.
__device__ __forceinline__ void dma16(const unsigned char* base_uniform, unsigned off, unsigned lds_base_uniform) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base_uniform), "s"(lds_base_uniform)
               : "memory", "m0");
}
// Wait until at most N LDS reads are outstanding (compiler-visible, so that it adds none of its own
// for fragments covered by this wait).  gfx9 encoding: vmcnt and expcnt left at their maxima.
template <int N>
__device__ __forceinline__ void wait_lds() {
  __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// MFMA issued by hand so that the register files are under control: S^T accumulates in VGPRs
// (the vector ALU reads it next), O^T in AGPRs, and the Q fragments (B operands) and the K
// fragments (A operands, loaded from LDS straight into AGPRs) sit in AGPRs too.
// The compiler does not see these as matrix instructions, so the read-after-MFMA-write distances
// the hardware needs are kept by construction (see mfma_settle_*()).
__device__ __forceinline__ void mfma_qk_first(floatx16& s, const bf16x8& a, const bf16x8& q, const floatx16& c0) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %3" : "=&v"(s) : "a"(a), "a"(q), "v"(c0));
}
__device__ __forceinline__ void mfma_qk(floatx16& s, const bf16x8& a, const bf16x8& q) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(s) : "a"(a), "a"(q));
}
__device__ __forceinline__ void mfma_pv(floatx16& o, const bf16x8& a, const bf16x8& pfrag) {
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(o) : "v"(a), "v"(pfrag));
}
// 48 idle issue cycles tied to a register tuple: everything that reads or writes `x` afterwards
// is ordered behind a finished matrix pipe (an 8-pass MFMA result is readable 19 cycles after issue).
__device__ __forceinline__ void mfma_settle_v(floatx16& x) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+v"(x));
}
__device__ __forceinline__ void mfma_settle_a(floatx16& x) {
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" : "+a"(x));
}

// V ring slots (the K ring has one more): three for the two-unit kernel, one workgroup per CU, 112 KB of
// LDS; two for the one-unit kernel so that two workgroups share a CU's 160 KB.  A deeper ring bought
// nothing in measurements, neither on L2-resident prefixes nor on HBM-bound decode-shaped steps.
constexpr int kRingTwoUnits = 3, kRingOneUnit = 2;
constexpr float kRescaleThreshold = 16.0f;  // log2 units: stale running max tolerated up to 2^16
constexpr float kSumThreshold = 1048576.0f;             // 2^20: row sum of a half that moves the reference up
constexpr float kRedoThreshold = 1152921504606846976.0f;  // 2^60: beyond this the workgroup starts over

// Slot schedule of one pipeline step of a wavefront with QA active units (QA = QB in the ordinary
// step; QA = 1 in a two-unit wavefront whose first unit has passed its causal horizon).  A step
// handles one 32-key half hh and consists of M MFMA slots: M1 slots forming S^T of half hh+1 (phase
// 1), then M2 slots accumulating O^T += V^T P^T of half hh (phase 2).  A single wavefront hides only
// about 16-20 cycles of other instructions under one 32-cycle MFMA (an exp2 costs 8, plain vector
// instructions 4), so everything else is dealt out evenly, a fixed share behind every MFMA:
//   * exp2 / pack / row-sum "events" of half hh (one event = one exp2; the second event of a logit
//     pair also packs the pair, and each event adds the exp2 before it to the row sum): events
//     [NEAR, NE) in slots [0, EW) of the half's own step, so that slab 0 of P is packed before phase
//     2 and slab 1 before its second half; with SUM_MODE the first NEAR events (all in slab 0) are
//     taken EARLY, in the tail slots [EW, M) of the step before, as soon as that S^T is complete;
//   * LDS fragment reads one batch ahead, in slots [0, RW), RW half way into the tail, one wait per batch;
//   * SUM_MODE: the test of the row sums against 2^20 right after the last event; else the row
//     maxima of half hh+1 and the rescale decision in the exp-free tail [RM0, M);
//   * in odd steps the workgroup barrier and the ring refill (DMA) in the tail [EW, M).
template <int D, int QA, bool SUM_MODE, int LPG>
struct Sched {
  static constexpr int KS = D / 16, DB = D / 32;
  static constexpr int M1 = KS * QA;       // MFMAs of phase 1 (K fragment ks feeds QA of them)
  static constexpr int M2 = 2 * DB * QA;   // MFMAs of phase 2 (V^T fragment (tt, db) feeds QA of them)
  static constexpr int M = M1 + M2;
  static constexpr int NP = QA * 8;        // logit pairs per step; pair k: slab k / (4 QA), unit (k / 4) % QA
  static constexpr int NE = 2 * NP;        // exp events
  static constexpr int EW = M1 + M2 / 2;
  static constexpr int NEAR = SUM_MODE ? (NE * (M - EW) / M) & ~1 : 0;
  static constexpr int NMAIN = NE - NEAR;
  static_assert(NEAR <= NE / 2, "early events must stay inside slab 0");
  static_assert(NEAR + (M1 * NMAIN + EW - 1) / EW >= NE / 2, "slab 0 would not be complete at the start of phase 2");
  static constexpr int GK = KS / 2;        // K fragments per batch (two batches per step)
  static constexpr int GV = DB;            // V^T fragments per batch (two batches per step, 2 reads each)
  static constexpr int R = 2 * GK + 4 * GV;  // LDS read instructions per step, in issue order:
                                             //   kg[1] (GK) | vg[0] (2 GV) | vg[1] (2 GV) | kg[0] of the next step (GK)
  static constexpr int RW = EW + (M - EW) / 2;  // (measured: spreading the reads a little into the tail beats stopping at EW)
  static_assert(EW + 1 < M, "no slot for the row-sum test");
  static constexpr int RM1 = M - 1 - QA;   // row-max slots [RM0, RM1), then QA + 1 decision slots
  static constexpr int RM0 = (EW - (M >= 32 ? 2 : 0)) < RM1 ? (EW - (M >= 32 ? 2 : 0)) : RM1 - 1;
  static_assert(SUM_MODE || RM0 >= M1 + 1, "row maxima would read S^T before its MFMAs retire");
  static_assert(SUM_MODE || (RM1 > RM0 && RM1 + QA < M), "no room for the row maxima");
  static_assert(LPG <= (M - EW) * 4, "ring refill does not fit the tail");
  // read r is issued in slot r * RW / R; reads issued before slot sl:
  static constexpr int rd_before(int sl) {
    int n = 0;
    for (int r = 0; r < R; ++r) n += (r * RW / R) < sl;
    return n;
  }
};

template <int D, int QB, int NV>
__global__ void __launch_bounds__(256, (QB == 1 ? 2 : 1)) attn_bf16_kernel(AttnParams p) {
  // Sum-driven reference updates (no row max below the causal horizon) for the two-unit kernel, whose
  // single wavefront per SIMD cannot hide the row-max work; the one-unit kernel has a second
  // wavefront to hide it and fewer registers, and takes the exact row max of every half.
  constexpr bool SUM_MODE = QB == 2;
  extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
  const unsigned lds0 = (unsigned)(uintptr_t)((unsigned char __attribute__((address_space(3)))*)smem);
  constexpr int NK = NV + 1;         // K ring slots (K runs half a tile ahead of V in the pipeline)
  constexpr int CH = D / 8;          // 16-byte chunks per row
  constexpr int ROWB = D * 2;        // bytes per row
  constexpr int BN = kTileKeys;      // 64
  constexpr int KS = D / 16;         // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;         // 32-wide blocks of the head dim in O^T
  constexpr int TILEB = BN * ROWB;   // bytes of one K (or V) tile
  constexpr int HALFB = 32 * ROWB;   // bytes of a 32-key half tile
  constexpr int RPS = 64 / CH;       // rows covered by one 1 KiB DMA slab
  constexpr int SLABS = CH / 4;      // slabs per wavefront per tensor per tile
  constexpr int LPG = 2 * SLABS;     // DMA instructions per wavefront per tile (K + V)
  constexpr int KSW = CH < 16 ? CH : 16;  // K swizzle: chunk ^= row % KSW
  constexpr int VSW = CH / 4;             // V swizzle: chunk ^= (row & 3) * VSW

  // rings: K slots [0, NK), V slots [NK, NK + NV)

  // ---- which workgroup am I (XCD-aware: a KV head stays on its XCDs, see logical_workgroup())
  const int wgs_per_kvh = p.wgs_per_head * p.n_splits;
  const int lid = logical_workgroup((int)blockIdx.x, (int)gridDim.x, p.n_q_heads / p.group, wgs_per_kvh);
  if (lid >= p.n_wgs) return;
  const int g = lid / wgs_per_kvh;
  const int rem = lid - g * wgs_per_kvh;
  const int split = rem / p.wgs_per_head;
  // Later token blocks see more keys.  Default order: heaviest first (longest-processing-time
  // first over several rounds of workgroups).  With pair_order the grid is resident at once, two
  // workgroups per CU, dispatched in id order: the first half descends from the heaviest, the second
  // half ascends from the lightest, so the two workgroups that share a CU add up to the same work.
  int ug;
  {
    const int idx = rem - split * p.wgs_per_head, W = p.wgs_per_head, half = (W + 1) / 2;
    ug = (!p.pair_order || idx < half) ? W - 1 - idx : idx - half;
  }

  const int tid = threadIdx.x, l = tid & 63, hi = l >> 5, m = l & 31;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int C = p.n_tokens, Hq = p.n_q_heads, G = p.group;
  const int Lm1 = (int)(p.len_prev + C - 1);  // last valid cache row
  constexpr int UPW = kUnitsPerWg * QB;        // units per workgroup
  const float sc = p.scale_log2e;

  // ---- my units
  int tok[QB], head[QB], tokc[QB];
  bool store_ok[QB], unit_valid[QB];
  int my_vis[QB];     // keys visible to this lane's query row
  int vis_first[QB];  // keys visible to the unit's first row (key blocks entirely below need no mask)
  int vis_last0 = 0;  // keys visible to the last row of unit 0: tiles entirely beyond are dead for it
  // Sink + sliding-window step (Sec. 6 of the paper, the streaming baseline's mask): the row that sees keys
  // [0, vis) sees of them only j < n_sink and j >= vis - window.  lb_last: the largest such lower bound among
  // the rows of the wavefront's units; key blocks that begin below it need the left mask.
  const bool win = p.window > 0;
  const int n_sink = p.n_sink;
  int lb_last = 0;
  // pair_units (two-unit kernel): wavefront number n = 4 ug + w of the KV head owns unit n, counted from
  // the first token block, and unit U-1-n, counted from the last, so that every wavefront has the
  // same number of (row, key) pairs to do whatever the causal horizon; else units 2n and 2n+1.
  const bool pair_units = QB == 2 && p.pair_units;
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const int n = ug * kUnitsPerWg + w;
    const int u = !pair_units ? n * QB + qb : (qb == 0 ? n : p.units_per_head - 1 - n);
    const bool valid = !pair_units ? u < p.units_per_head : (qb == 0 ? 2 * n <= p.units_per_head - 1 : 2 * n < p.units_per_head - 1);
    const int uc = u < 0 ? 0 : (u < p.units_per_head ? u : p.units_per_head - 1);
    const int tb = uc / G, hg = uc - tb * G;
    head[qb] = g * G + hg;
    tok[qb] = tb * kRowsPerUnit + m;
    tokc[qb] = tok[qb] < C ? tok[qb] : C - 1;
    unit_valid[qb] = valid;
    store_ok[qb] = valid && (tok[qb] < C);
    {
      const int last = tb * kRowsPerUnit + kRowsPerUnit - 1;
      const int vis_last = (int)p.len_prev + (last < C ? last : C - 1) + 1;
      if (qb == 0) vis_last0 = vis_last;
      if (win && vis_last - p.window > lb_last) lb_last = vis_last - p.window;
    }
    my_vis[qb] = (int)p.len_prev + tokc[qb] + 1;
    vis_first[qb] = (int)p.len_prev + tb * kRowsPerUnit + 1;
  }
  const int vis_min = vis_first[0];  // units are ordered by token block, so unit 0 has the nearest horizon

  // ---- tile range of this workgroup / split
  int nkeys_wg;
  {
    // the unit of the workgroup with the farthest horizon: its last one, or with pair_units the partner of its first
    int ulast = pair_units ? p.units_per_head - 1 - ug * kUnitsPerWg : ug * UPW + UPW - 1;
    if (ulast > p.units_per_head - 1) ulast = p.units_per_head - 1;
    if (ulast < 0) ulast = 0;
    int row_hi = (ulast / G) * kRowsPerUnit + kRowsPerUnit - 1;
    if (row_hi > C - 1) row_hi = C - 1;
    nkeys_wg = (int)p.len_prev + row_hi + 1;
  }
  // logical tiles 0 .. ntiles-1 of this workgroup; under a window the tiles between the sinks and the window
  // are left out: logical tile t is physical tile t + (t >= ns_t ? skip : 0)
  TileMap tm;
  if (win) {
    const RowRange rr = workgroup_rows(ug, UPW, p.units_per_head, G, C);
    tm = tile_map(p.len_prev, rr.row_lo, rr.row_hi, n_sink, p.window);
  } else {
    tm.ns_t = 0;
    tm.skip = 0;
    tm.ntiles = (nkeys_wg + BN - 1) / BN;
  }
  const int ns_t = tm.ns_t, t_skip = tm.skip;
  auto tphys = [&](int t) __attribute__((always_inline)) -> int { return t + (t >= ns_t ? t_skip : 0); };
  // first logical tile whose physical tile is not below tp
  auto tlogical = [&](int tp) __attribute__((always_inline)) -> int {
    if (tp < ns_t) return tp;
    return tp - t_skip > ns_t ? tp - t_skip : ns_t;
  };
  // this workgroup's piece of them, and what its DMA may touch (shared with the host-side model of this walk)
  const KeyRange kr = key_range(tm, split, p.tiles_per_split, p.len_prev, C, p.k_new != nullptr);
  const int t_begin = kr.t_begin, t_end = kr.t_end;

  const unsigned char* kbase = reinterpret_cast<const unsigned char*>(p.k_cache) + (int64_t)g * p.capacity * ROWB;
  const unsigned char* vbase = reinterpret_cast<const unsigned char*>(p.v_cache) + (int64_t)g * p.capacity * ROWB;

  // ---- fused append (paper Sec. 2: the chunk's K/V rows join the cache): tiles from t_new on lie in the
  // chunk and are streamed from the rows as handed in, [C][Hkv][d], so no workgroup waits for another's
  // copy; the copy into the cache, for the steps to come, is shared out over the workgroups of the KV head.
  const bool fused = p.k_new != nullptr;
  const unsigned new_stride = (unsigned)(p.n_kv_heads * ROWB);  // bytes from one token's row to the next
  const unsigned char* knew = reinterpret_cast<const unsigned char*>(p.k_new) + (int64_t)g * ROWB;
  const unsigned char* vnew = reinterpret_cast<const unsigned char*>(p.v_new) + (int64_t)g * ROWB;
  // This workgroup's share of the copy: rows [r0, r1) of K and of V, 16 bytes per lane and access.  The first
  // kCopyFirst vectors per lane are only loaded here and stored once the ring refill and the Q loads are on
  // their way, so that their latency is not paid on its own; whatever is left (few workgroups, long chunks)
  // is copied on the spot.
  constexpr int kCopyFirst = 8;
  uintx4 copy_v[kCopyFirst];
  int copy_r0 = 0, copy_nvec = 0;
  auto copy_src = [&](int idx) __attribute__((always_inline)) -> const uintx4* {
    const bool is_v = idx >= copy_nvec;
    const int e = is_v ? idx - copy_nvec : idx, r = copy_r0 + e / CH, c = e % CH;
    return reinterpret_cast<const uintx4*>((is_v ? vnew : knew) + (int64_t)r * new_stride + c * 16);
  };
  auto copy_dst = [&](int idx) __attribute__((always_inline)) -> uintx4* {
    const bool is_v = idx >= copy_nvec;
    const int e = is_v ? idx - copy_nvec : idx, r = copy_r0 + e / CH, c = e % CH;
    return reinterpret_cast<uintx4*>(const_cast<unsigned char*>(is_v ? vbase : kbase) + (p.len_prev + r) * ROWB + c * 16);
  };
  if (fused) {
    const int per = (C + wgs_per_kvh - 1) / wgs_per_kvh;  // rows of this workgroup
    const int r1 = rem * per + per < C ? rem * per + per : C;
    copy_r0 = rem * per;
    copy_nvec = (r1 > copy_r0 ? r1 - copy_r0 : 0) * CH;  // 16-byte vectors per tensor
#pragma unroll
    for (int u = 0; u < kCopyFirst; ++u)
      if (tid + u * 256 < 2 * copy_nvec) copy_v[u] = *copy_src(tid + u * 256);
    for (int idx = tid + kCopyFirst * 256; idx < 2 * copy_nvec; idx += 256) __builtin_nontemporal_store(*copy_src(idx), copy_dst(idx));
  }

  // ---- DMA addressing: wavefront w moves slabs w, w+4, ...; lane l lands at chunk (l % CH) of row
  // slab*RPS + l / CH and therefore fetches the chunk that the swizzle maps there.  Offsets from
  // the head's base are 32-bit (the host checks capacity * row bytes < 2^32).
  const int dma_row0 = w * RPS + l / CH;  // + i * 4 * RPS for slab i
  const unsigned dma_kc = (unsigned)(((l % CH) ^ (dma_row0 % KSW)) * 16);
  const unsigned dma_vc = (unsigned)(((l % CH) ^ ((dma_row0 & 3) * VSW)) * 16);
  const unsigned dma_koff = (unsigned)dma_row0 * ROWB + dma_kc;  // lane part of an unclamped offset
  const unsigned dma_voff = (unsigned)dma_row0 * ROWB + dma_vc;
  // slab i of tile t of K (is_v = false) or V; CLAMP redirects rows past the cache end, or past this
  // workgroup's key range (the ring runs NV + 1 tiles ahead and knows no end), to the last row inside:
  // they are never used, and so are never fetched from HBM either
  // (kr.row_lim).  Fused append: tiles from kr.t_new on lie in the chunk -- unless this workgroup's key range ends
  // before the chunk begins: then every row past the range is redirected to row_lim, a cache row, whatever its tile.
  const int t_new = kr.t_straddle >= 0 ? kr.t_straddle : kr.t_new;  // first physical tile with rows of the chunk
  auto issue_slab = [&](bool is_v, int t_log, int slot, int i, auto clamp_tag, unsigned extra = 0) __attribute__((always_inline)) {
    constexpr bool CLAMP = decltype(clamp_tag)::value;
    const int t = tphys(t_log);
    const unsigned lds = lds0 + (unsigned)(((is_v ? NK : 0) + slot) * TILEB + (w + 4 * i) * 1024);
    unsigned off;
    if (CLAMP) {
      int row0_here = dma_row0;  // opaque copy: what is derived from it is computed here, not once ahead of all
      asm volatile("" : "+v"(row0_here));  // loops and then held in registers through the main loop
      const DmaRow src = dma_row(kr, t, row0_here + i * 4 * RPS);
      if (__builtin_expect(t != kr.t_straddle, 1)) {
        // (wave-uniform choice, scalar selects) a tile of the chunk itself comes from the rows as handed in
        const bool nw = t >= kr.t_new;
        const unsigned char* base = nw ? (is_v ? vnew : knew) : (is_v ? vbase : kbase);
        const unsigned stride = nw ? new_stride : (unsigned)ROWB;
        off = src.row * stride + (is_v ? dma_vc : dma_kc) + extra;
        dma16(base, off, lds);
      } else if (src.from_chunk) {
        // the one tile with rows on both sides of the cache's end (cache length not a multiple of the tile): each
        // lane fetches from its own side, two DMA instructions with complementary lanes fill the slab
        dma16(is_v ? vnew : knew, src.row * new_stride + (is_v ? dma_vc : dma_kc) + extra, lds);
      } else {
        dma16(is_v ? vbase : kbase, src.row * (unsigned)ROWB + (is_v ? dma_vc : dma_kc) + extra, lds);
      }
    } else {
      off = (is_v ? dma_voff : dma_koff) + (unsigned)(t * BN + i * 4 * RPS) * ROWB;
      dma16(is_v ? vbase : kbase, off, lds);
    }
  };
  auto issue_k = [&](int t, unsigned extra) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < SLABS; ++i) issue_slab(false, t, t % NK, i, std::true_type{}, extra);
  };
  auto issue_v = [&](int t, unsigned extra) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < SLABS; ++i) issue_slab(true, t, t % NV, i, std::true_type{}, extra);
  };

  // ---- the ring is filled first (only addresses are needed), then the Q fragments are fetched: the two
  // latencies overlap.  Q, pre-multiplied by scale*log2(e), stays in registers for the whole kernel.
  auto prefill = [&](unsigned extra) __attribute__((always_inline)) {
    // Steady state at the top of the even step of tile t: K[t], K[t+1], V[t] are in LDS and visible, the
    // groups {K[t+1+j], V[t+j]}, j = 1 .. NV-1, are in flight.
    issue_k(t_begin, extra);
    issue_k(t_begin + 1, extra);
    issue_v(t_begin, extra);
#pragma unroll
    for (int j = 1; j < NV; ++j) {
      issue_k(t_begin + 1 + j, extra);
      issue_v(t_begin + j, extra);
    }
  };
  if (t_begin < t_end) prefill(0u);
  bf16x8 qf[QB][KS];
  {
    bf16x8 raw[QB][KS];  // every load in flight before the first is waited for
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const __bf16* qrow = reinterpret_cast<const __bf16*>(p.q) + ((int64_t)tokc[qb] * Hq + head[qb]) * D;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) raw[qb][ks] = *reinterpret_cast<const bf16x8*>(qrow + ks * 16 + hi * 8);
    }
    if (fused) {
#pragma unroll
      for (int u = 0; u < kCopyFirst; ++u)
        if (tid + u * 256 < 2 * copy_nvec) __builtin_nontemporal_store(copy_v[u], copy_dst(tid + u * 256));
    }
    if (p.rope_cos) {
      // Rotary embedding at the row's absolute position (Sec. 2), half-split pairs (j, j + D/2), fp32 with
      // the sine product rounded first, result rounded to bf16: bit for bit what a caller that rotates q
      // itself and stores it as bf16 would hand in.  Fragments ks and ks + KS/2 hold the two halves of 8 pairs.
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int ks = 0; ks < KS / 2; ++ks) {
          const float* cs = p.rope_cos + (int64_t)tokc[qb] * (D / 2) + ks * 16 + hi * 8;
          const float* sn = p.rope_sin + (int64_t)tokc[qb] * (D / 2) + ks * 16 + hi * 8;
          const bf16x8 lo = raw[qb][ks], up = raw[qb][ks + KS / 2];
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            const float tl = (float)up[e] * sn[e], tu = (float)lo[e] * sn[e];
            raw[qb][ks][e] = (__bf16)__builtin_fmaf((float)lo[e], cs[e], -tl);
            raw[qb][ks + KS / 2][e] = (__bf16)__builtin_fmaf((float)up[e], cs[e], tu);
          }
        }
      }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[qb][ks][e] = (__bf16)((float)raw[qb][ks][e] * sc);
        asm volatile("" : "+a"(qf[qb][ks]));  // park the fragment in the AGPR file, where the MFMAs read it
      }
  }

  // ---- LDS read offsets (per lane) of the tile currently being read, ring slot included; moved
  // from slot to slot once per tile
  // K fragment (A operand of S^T): row kb*32+m, chunk ks*2+hi, swizzled by row % KSW = m % KSW
  int kslot, vslot;  // ring slots of tile t (wave-uniform)
  unsigned kaddr[KS];
  unsigned vaddr[DB];

  // ---- running state
  floatx16 o[QB][DB];   // O^T accumulators (AGPRs)
  floatx16 negm[QB];    // -m (0 while no key has been seen) in every element: start value of S^T
  float m_run[QB], l_run[QB];
  int overflowed = 0;   // wave-uniform: a row sum left the range the sum-driven rescale can repair
  auto reset_state = [&]() __attribute__((always_inline)) {
    kslot = t_begin % NK;
    vslot = t_begin % NV;
    // derived from an opaque copy of the lane id, so that nothing computed here is kept in registers
    // across the main loop for the sake of a restart that almost never happens
    int l2 = l;
    asm volatile("" : "+v"(l2));
    const int hi2 = l2 >> 5, m2 = l2 & 31;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      kaddr[ks] = lds0 + (unsigned)(m2 * ROWB + (((ks * 2 + hi2) ^ (m2 % KSW)) * 16)) + (unsigned)(kslot * TILEB);
    // V^T fragment via transpose read: lane i of a 16-lane block supplies row (i/4) of a 4-row group and 4 columns
    const int i16 = l2 & 15, b2 = (l2 >> 4) & 1;
    const int v_row = 4 * hi2 + (i16 >> 2);  // + 16*tt (+8)
#pragma unroll
    for (int db = 0; db < DB; ++db)
      vaddr[db] = lds0 + (unsigned)(v_row * ROWB + (((4 * db + 2 * b2 + ((i16 & 3) >> 1)) ^ ((v_row & 3) * VSW)) * 16) + 8 * (i16 & 1)) +
                  (unsigned)((NK + vslot) * TILEB);
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      m_run[qb] = -INFINITY;
      l_run[qb] = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) negm[qb][r] = 0.f;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qb][db][r] = 0.f;
    }
  };

  // ---- building blocks of the software pipeline --------------------------------------------
  // K fragment ks of the current K tile (imm = 0) or of its second half (imm = HALFB), read from LDS
  // straight into AGPRs.  The compiler does not see an LDS access here: every use is covered by one
  // of the wait_lds<>() calls of the pipeline.
  auto k_frag = [&](int ks, int imm) __attribute__((always_inline)) -> bf16x8 {
    bf16x8 f;
    if (imm == 0)
      asm volatile("ds_read_b128 %0, %1" : "=a"(f) : "v"(kaddr[ks]));
    else
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=a"(f) : "v"(kaddr[ks]), "n"(HALFB));
    return f;
  };
  // causal mask (and, under a window, the mask of the keys between the sinks and the window) of the 32-key
  // half hh (logical numbering)
  auto mask_half = [&](floatx16 (&s)[QB], int hh, int q0 = 0) __attribute__((always_inline)) {
    // (opaque copies: whatever is derived from them is computed here, not once ahead of all loops and
    // then held in registers through the unmasked main loop)
    int hi_here = hi;
    asm volatile("" : "+v"(hi_here));
    const int key0 = (2 * tphys(hh >> 1) + (hh & 1)) * 32;  // first key of the half
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (qb < q0) continue;
      if (key0 + 32 > vis_first[qb]) {  // wave-uniform
        int vis_here = my_vis[qb];
        asm volatile("" : "+v"(vis_here));
        const int rel = vis_here - key0;
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (8 * (r >> 2) + 4 * hi_here + (r & 3) >= rel) s[qb][r] = -INFINITY;
      }
      if (win && key0 < lb_last && key0 + 32 > n_sink) {  // wave-uniform
        int vis_here = my_vis[qb];
        asm volatile("" : "+v"(vis_here));
        const int rel_lb = vis_here - p.window - key0, rel_sink = n_sink - key0;  // visible: below rel_sink or from rel_lb on
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kk = 8 * (r >> 2) + 4 * hi_here + (r & 3);
          if (kk < rel_lb && kk >= rel_sink) s[qb][r] = -INFINITY;
        }
      }
    }
  };
  // mx[] holds the row maxima of a half whose logits are already relative to the running max, i.e.
  // by how much the max would grow.  The running max is raised only when it lags by more than
  // 2^16 (or has never been set).  The decision (cross-lane max, compare) is taken early, under
  // the matrix pipe; the branch comes later.
  auto rescale_need = [&](const float (&dm)[QB], int q0 = 0) __attribute__((always_inline)) -> bool {
    int need = 0;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)  // no short-circuit: plain lane-wise compares, one wave-wide reduction at the end
      if (qb >= q0) need |= (int)(dm[qb] > kRescaleThreshold) | ((int)(m_run[qb] == -INFINITY) & (int)(dm[qb] > -INFINITY));
    return __any(need);
  };
  auto rescale_decide = [&](const float (&mx)[QB], float (&dm)[QB], int q0 = 0) __attribute__((always_inline)) -> bool {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
      if (qb >= q0) dm[qb] = pair_max(mx[qb]);
    return rescale_need(dm, q0);
  };
  // s holds the logits of the half the maxima came from: they were formed against the old max
  auto rescale_apply = [&](const float (&dm)[QB], floatx16 (&s)[QB], int q0 = 0) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (qb < q0) continue;
      const float cur = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
      // only rows that asked for it move, so a row's arithmetic never depends on its wave neighbours
      const bool mine = (dm[qb] > kRescaleThreshold) || (m_run[qb] == -INFINITY && dm[qb] > -INFINITY);
      const float m2 = mine ? fmaxf(m_run[qb], cur + dm[qb]) : m_run[qb];
      const float use = (m2 == -INFINITY) ? 0.f : m2;
      const float delta = use - cur;
      // a row without history (l = 0, O = 0) has nothing to scale, and its first reference may lie far enough
      // below zero for 2^-delta to overflow
      const float alpha = (m_run[qb] == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f(-delta);
      m_run[qb] = m2;
      l_run[qb] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        negm[qb][r] = -use;
        s[qb][r] -= delta;
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        mfma_settle_a(o[qb][db]);
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
      }
    }
  };
  // The first half of a pass: no history, so the row max of the half is the reference (0 for a row that sees
  // none of its keys) and neither l nor O needs touching.
  auto reference_first = [&](const float (&mx)[QB], floatx16 (&s)[QB]) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      const float dm = pair_max(mx[qb]);
      const float use = (dm > -INFINITY) ? dm : 0.f;
      m_run[qb] = dm;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        negm[qb][r] = -use;
        s[qb][r] -= use;
      }
      asm volatile("" : "+v"(negm[qb]));  // 16 registers from here on, not one value splatted anew ahead of every MFMA chain
    }
  };
  // ls[] holds the row sums of the half just exponentiated (per lane: the 16 keys it owns).  A sum
  // above 2^20 moves the reference up by the power of two just above it, which is exact; s holds
  // the in-flight logits of the next half, formed against the old reference.  Both lanes of a row
  // decide on the larger of their two sums, so a row never depends on its wave neighbours.
  auto rescale_from_sum = [&](const float (&ls)[QB], floatx16 (&s)[QB], int q0 = 0) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (qb < q0) continue;
      const float tot = pair_max(ls[qb]);
      const bool bad = !(tot <= kRedoThreshold);  // also infinite or NaN
      overflowed |= __any((int)bad);
      const bool mine = !(tot <= kSumThreshold) && !bad;
      const int e = mine ? __builtin_amdgcn_frexp_expf(tot) : 0;  // tot < 2^e
      const float delta = (float)e;
      const float alpha = __builtin_ldexpf(1.0f, -e);
      const float cur = (m_run[qb] == -INFINITY) ? 0.f : m_run[qb];
      const float use = cur + delta;
      if (mine) m_run[qb] = use;
      l_run[qb] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        negm[qb][r] = -use;
        s[qb][r] -= delta;
      }
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        mfma_settle_a(o[qb][db]);
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qb][db][r] *= alpha;
      }
    }
  };
  auto rowmax_all = [&](floatx16 (&s)[QB], float (&mx)[QB], int q0 = 0) __attribute__((always_inline)) {
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      if (qb < q0) continue;
      float a = fmaxf(s[qb][0], s[qb][1]);
#pragma unroll
      for (int r = 2; r < 16; r += 2) a = fmaxf(fmaxf(a, s[qb][r]), s[qb][r + 1]);
      mx[qb] = a;
    }
  };

  // ---- the software pipeline (slot schedule: struct Sched) -----------------------------------
  constexpr int GK = KS / 2, GV = DB;  // fragments per batch, whatever the number of active units

  floatx16 sA[QB], sB[QB];
  uintx4 pb[QB][2];      // P^T fragments: 8 bf16 per 16-key slab, as packed pairs
  float lsum_early[QB];  // row sums of the early events of the half that the next step finishes
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) lsum_early[qb] = 0.f;
  // One exp event of a half whose logits are in s: event j covers logit j of the half's 2 NP, in
  // pairs; the second event of a pair also packs the pair into its P^T slot and the first adds the
  // previous pair's second exp to the row sum (`first`: there is none pending).
  float ev_a = 0.f, ev_b = 0.f;  // first exp of the pair in flight; second exp not yet in its row sum
  // unit that event j of a step with units Q0 .. QB-1 belongs to
  auto ev_unit = [](int j, int Q0, int QA) constexpr { return Q0 + (((j >> 1) % (QA * 4)) >> 2); };
  auto exp_event = [&](const floatx16 (&s)[QB], float (&ls)[QB], int j, bool first, auto q0_tag) __attribute__((always_inline)) {
    constexpr int Q0 = decltype(q0_tag)::value, QA = QB - Q0;  // active units Q0 .. QB-1
    const int k = j >> 1, slab = k / (QA * 4), kk = k % (QA * 4);
    const int qb = Q0 + (kk >> 2), jj = kk & 3, r = 8 * slab + 2 * jj;
    if ((j & 1) == 0) {
      if (first)
        asm volatile("v_exp_f32_e32 %0, %1" : "=v"(ev_a) : "v"(s[qb][r]));
      else
        asm volatile(
            "v_exp_f32_e32 %0, %2\n\t"
            "v_add_f32_e32 %1, %3, %1"
            : "=&v"(ev_a), "+v"(ls[ev_unit(j - 1, Q0, QA)])
            : "v"(s[qb][r]), "v"(ev_b));
    } else {
      float eb;
      unsigned pku;
      asm volatile(
          "v_exp_f32_e32 %0, %3\n\t"
          "v_add_f32_e32 %2, %4, %2\n\t"
          "v_cvt_pk_bf16_f32 %1, %4, %0"
          : "=&v"(eb), "=v"(pku), "+v"(ls[qb])
          : "v"(s[qb][r + 1]), "v"(ev_a));
      pb[qb][slab][jj] = pku;
      ev_b = eb;
    }
  };
  // the early events of a half all at once (prologue, masked steps, and again after a sum-driven shift)
  auto early_events = [&](const floatx16 (&s)[QB], auto q0_tag) __attribute__((always_inline)) {
    constexpr int Q0 = decltype(q0_tag)::value, QA = QB - Q0;
    constexpr int NEAR = Sched<D, QA, SUM_MODE, LPG>::NEAR;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) lsum_early[qb] = 0.f;
    if (NEAR > 0) {
#pragma unroll
      for (int j = 0; j < NEAR; ++j) exp_event(s, lsum_early, j, j == 0, q0_tag);
      lsum_early[ev_unit(NEAR - 1, Q0, QA)] += ev_b;
    }
  };
  bf16x8 kg[2][GK];          // K fragment batches
  short4_ vh[2][GV][2];      // V^T fragment batches, as the two transpose-read halves of each fragment
  auto v_half = [&](int tt, int db, int half, int imm) __attribute__((always_inline)) -> short4_ {
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4_, vaddr[db] + (unsigned)(imm + 16 * tt * ROWB + half * 8 * ROWB)));
  };

  // One pipeline step for half hh.  On entry s_cur holds S^T of half hh (masked, relative to the
  // running max), kg[0] the first batch of K fragments of half hh+1, and kaddr/vaddr point at the
  // tiles of halves hh+1 / hh.  ODD steps (second half of a tile) end with the workgroup barrier
  // and the ring refill for the tiles after next; MASKED selects the variant for halves hh+1 that
  // reach past the causal horizon, and for every half once a row sum has overflowed (mask, then the
  // exact row max, after the matrix work); CLAMP the variant whose refill may run past the end of
  // the cache.  q0_tag = 1 (two-unit kernel only): unit 0 has passed its causal horizon for good and
  // only unit 1 is worked on, with the schedule of a one-unit step; a masked step of both units that
  // is followed by such a step (next_unit1_only) leaves the early events in that step's numbering.
  auto step = [&](floatx16 (&s_cur)[QB], floatx16 (&s_next)[QB], int hh, auto odd_tag, auto masked_tag,
                  auto clamp_tag, auto q0_tag, bool next_unit1_only = false) __attribute__((always_inline)) {
    constexpr bool ODD = decltype(odd_tag)::value;
    constexpr bool MASKED = decltype(masked_tag)::value;
    constexpr int Q0 = decltype(q0_tag)::value, QA = QB - Q0;
    using S = Sched<D, QA, SUM_MODE, LPG>;
    constexpr int M1 = S::M1, M = S::M, EW = S::EW, NE = S::NE, NEAR = S::NEAR, NMAIN = S::NMAIN, NP = S::NP;
    constexpr int R = S::R, RW = S::RW, RM0 = S::RM0, RM1 = S::RM1;
    const int t = hh >> 1;
    constexpr int KIMM = ODD ? 0 : HALFB;  // even hh: half hh+1 is the second half of tile t
    constexpr int VIMM = ODD ? HALFB : 0;  // even hh: half hh is the first half of tile t
    float lsum[QB], lsum_next[QB];  // row sums of half hh (early part included) and of the early part of hh+1
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
      lsum[qb] = lsum_early[qb];
      lsum_next[qb] = 0.f;
    }  // (entries of units before Q0 are carried along untouched and never added anywhere)
    float mx[QB], dm[QB];
    bool need_rescale = false;
    int sum_flag = 0;      // per lane: a row sum of this half passed 2^20 (or is not a number)
    int kslot_prev = 0, vslot_prev = 0;

    wait_lds<0>();  // kg[0] (fetched at the end of the previous step) has landed
#pragma unroll
    for (int i = 0; i < M; ++i) {
      // ---- waits and the barrier come before the MFMA of the slot
      if (i == GK * QA) wait_lds<(S::rd_before(GK * QA) - GK)>();                 // kg[1]
      if (i == M1) wait_lds<(S::rd_before(M1) - GK - 2 * GV)>();                  // vg[0]
      if (i == EW) wait_lds<(S::rd_before(EW) - GK - 4 * GV)>();                  // vg[1]
      if (ODD && i == EW) {
        // Every read of K[t] and V[t] by this wave has returned.  K[t+2] and V[t+1] were issued
        // NV-1 tiles ago: they are the oldest group in flight.
        wait_vm<(NV - 2) * LPG>();
        __builtin_amdgcn_s_barrier();  // ... and this holds for every wave of the workgroup
        kslot_prev = kslot == 0 ? NK - 1 : kslot - 1;  // K[t]'s slot (kslot already names K[t+1]) takes K[t+1+NV]
        vslot_prev = vslot;                            // V[t]'s slot takes V[t+NV]
      }
      // ---- the MFMA
      if (i < M1) {
        const int ks = i / QA, qb = Q0 + i % QA;
        if (ks == 0)
          mfma_qk_first(s_next[qb], kg[0][0], qf[qb][0], negm[qb]);
        else
          mfma_qk(s_next[qb], kg[ks / GK][ks % GK], qf[qb][ks]);
      } else {
        const int sl = (i - M1) / QA, qb = Q0 + (i - M1) % QA, tt = sl / DB, db = sl % DB;
        const short8_ a8 = __builtin_shufflevector(vh[sl / GV][sl % GV][0], vh[sl / GV][sl % GV][1], 0, 1, 2, 3, 4, 5, 6, 7);
        mfma_pv(o[qb][db], __builtin_bit_cast(bf16x8, a8), __builtin_bit_cast(bf16x8, pb[qb][tt]));
      }
      __builtin_amdgcn_sched_barrier(0);
      // ---- its share of everything else
      // LDS reads
#pragma unroll
      for (int r = (i * R + RW - 1) / RW; r < ((i + 1) * R + RW - 1) / RW && r < R; ++r) {  // rd_slot(r) == i
        if (r < GK) {
          kg[1][r] = k_frag(GK + r, KIMM);
        } else if (r < GK + 4 * GV) {
          const int q = r - GK, f = q / 2, half = q % 2;  // fragment f = (tt, db) of the half, in use order
          vh[f / GV][f % GV][half] = v_half(f / DB, f % DB, half, VIMM);
        } else {
          const int j = r - GK - 4 * GV;
          kg[0][j] = k_frag(j, ODD ? HALFB : 0);  // kg[0] of the NEXT step (half hh+2)
        }
      }
      // after an even step the next K half starts a new tile: move the K read offsets to its ring
      // slot, a few per slot, between the last read of this tile's K and the first of the next
      if (!ODD && i >= GK * QA && i < GK * QA + (KS + 1) / 2) {
        const int kn = kslot + 1 == NK ? 0 : kslot + 1;
        const unsigned dk = (unsigned)((kn - kslot) * TILEB);
        const int a = (i - GK * QA) * 2;
        kaddr[a] += dk;
        if (a + 1 < KS) kaddr[a + 1] += dk;
        if (i == GK * QA + (KS + 1) / 2 - 1) kslot = kn;
      }
      // exp events of half hh ...
      if (i == EW) lsum[ev_unit(NE - 1, Q0, QA)] += ev_b;
#pragma unroll
      for (int j = NEAR + (i * NMAIN + EW - 1) / EW; j < NEAR + ((i + 1) * NMAIN + EW - 1) / EW && j < NE; ++j)
        exp_event(s_cur, lsum, j, j == NEAR, q0_tag);
      // ... and, below the causal horizon, the early ones of half hh+1, whose S^T is complete by now
      if (!MASKED && NEAR > 0 && i >= EW) {
#pragma unroll
        for (int j = ((i - EW) * NEAR + (M - EW) - 1) / (M - EW); j < ((i - EW + 1) * NEAR + (M - EW) - 1) / (M - EW) && j < NEAR; ++j)
          exp_event(s_next, lsum_next, j, j == 0, q0_tag);
        if (i == M - 1) lsum_next[ev_unit(NEAR - 1, Q0, QA)] += ev_b;
      }
      if (SUM_MODE && i == EW + 1) {
#pragma unroll
        for (int qb = Q0; qb < QB; ++qb) sum_flag |= (int)!(lsum[qb] <= kSumThreshold);
      }
      // row maxima of half hh+1 (its last MFMA is at least RM0 - M1 slots old), then the decision
      if (!SUM_MODE && !MASKED && i >= RM0 && i < RM1) {
#pragma unroll
        for (int k = ((i - RM0) * NP) / (RM1 - RM0); k < ((i - RM0 + 1) * NP) / (RM1 - RM0); ++k) {
          const int q2 = Q0 + (k >> 3), r = 2 * (k & 7);
          if (r == 0)
            mx[q2] = fmaxf(s_next[q2][0], s_next[q2][1]);
          else
            mx[q2] = fmaxf(fmaxf(mx[q2], s_next[q2][r]), s_next[q2][r + 1]);
        }
      }
      if (!SUM_MODE && !MASKED && i >= RM1 && i < RM1 + QA) dm[Q0 + i - RM1] = pair_max(mx[Q0 + i - RM1]);
      if (!SUM_MODE && !MASKED && i == RM1 + QA) need_rescale = rescale_need(dm, Q0);
      // ring refill and the V address of the next tile (odd steps, after the barrier)
      if (ODD && i >= EW) {
#pragma unroll
        for (int d = ((i - EW) * LPG) / (M - EW); d < ((i - EW + 1) * LPG) / (M - EW); ++d) {
          if (d < SLABS) issue_slab(false, t + 1 + NV, kslot_prev, d, clamp_tag);
          else issue_slab(true, t + NV, vslot_prev, d - SLABS, clamp_tag);
        }
        if (i == M - 1) {
          const int vn = vslot + 1 == NV ? 0 : vslot + 1;
          const unsigned dv = (unsigned)((vn - vslot) * TILEB);
#pragma unroll
          for (int d2 = 0; d2 < DB; ++d2) vaddr[d2] += dv;
          vslot = vn;
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int qb = Q0; qb < QB; ++qb) {
      l_run[qb] += lsum[qb];
      lsum_early[qb] = lsum_next[qb];
    }
    if constexpr (SUM_MODE) {
      if (__builtin_expect(__any(sum_flag), 0)) {
#pragma unroll
        for (int qb = Q0; qb < QB; ++qb) mfma_settle_v(s_next[qb]);
        rescale_from_sum(lsum, s_next, Q0);
        if (!MASKED) early_events(s_next, q0_tag);  // they were formed against the old reference: once more
      }
    }
    if (MASKED) {
#pragma unroll
      for (int qb = Q0; qb < QB; ++qb) mfma_settle_v(s_next[qb]);
      mask_half(s_next, hh + 1, Q0);
      rowmax_all(s_next, mx, Q0);
      need_rescale = rescale_decide(mx, dm, Q0);
    }
    if (__builtin_expect(need_rescale, 0)) {
#pragma unroll
      for (int qb = Q0; qb < QB; ++qb) mfma_settle_v(s_next[qb]);
      rescale_apply(dm, s_next, Q0);
    }
    if (MASKED) {
      if (QB == 2 && Q0 == 0 && next_unit1_only)
        early_events(s_next, std::integral_constant<int, QB - 1>{});
      else
        early_events(s_next, q0_tag);
    }
  };

  if (t_begin < t_end) {
    // A second pass (exact = true) follows only if a row sum overflowed in the first.
    for (bool exact = false;; exact = true) {
      reset_state();
      // Tiles whose two steps only produce halves entirely below the nearest causal horizon take the
      // fast variant: step 2t+1 produces half 2t+2 = keys [64t+64, 64t+96), so it needs 64t+96 <= vis_min.
      // (tile bounds are worked out on physical tiles, i.e. on keys, and then turned into logical tile numbers)
      int t_fast = tlogical((vis_min - 96) / BN + 1);  // first tile that is not fast (vis_min >= 1)
      if (vis_min < 96 || exact) t_fast = 0;
      if (t_fast > t_end) t_fast = t_end;
      // ... and tiles whose refill (tile t + 1 + NV) lies entirely inside the cache and the key range need no row
      // clamp (inside the cache proper when the append is fused)
      int t_nc = tlogical((Lm1 + 1) / BN < t_new ? (Lm1 + 1) / BN : t_new) - NV - 1;
      if (t_nc > t_end - NV - 1) t_nc = t_end - NV - 1;
      if (t_nc > t_fast) t_nc = t_fast;
      // Under a window the first tiles (the sinks, and the tiles that begin below the window of the wavefront's
      // last row) are masked on the left: tiles [t_begin, t_lead) take the masked variant
      int t_lead = win ? tlogical((lb_last + BN - 1) / BN) : 0;
      if (win && t_lead < ns_t) t_lead = ns_t;
      if (t_lead > t_end) t_lead = t_end;
      // Two-unit kernel: from tile t_dead on every key is beyond the last row of unit 0 and only unit 1
      // is worked on, fast up to its own horizon (t_fast1), masked from there.
      int t_dead = tlogical((vis_last0 + BN - 1) / BN);
      if (t_dead < t_lead) t_dead = t_lead;
      if (QB == 1 || exact || t_dead > t_end) t_dead = t_end;
      int t_fast1 = tlogical((vis_first[QB - 1] - 96) / BN + 1);
      if (vis_first[QB - 1] < 96 || exact) t_fast1 = 0;
      if (t_fast1 < t_dead) t_fast1 = t_dead;
      if (t_fast1 > t_end) t_fast1 = t_end;
      // Prologue.  The first pass finds the ring filled ahead of the Q loads; a second pass fills it again.
      if (exact) {
        unsigned again_zero = 0;  // opaque zero: keeps these addresses from being computed once and held in
        asm volatile("" : "+v"(again_zero));  // registers across the main loop for the sake of a second pass
        prefill(again_zero);
      }
      wait_vm<(NV - 1) * LPG>();
      __builtin_amdgcn_s_barrier();
      {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kg[ks / GK][ks % GK] = k_frag(ks, 0);
        wait_lds<0>();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
          for (int qb = 0; qb < QB; ++qb) {
            if (ks == 0)
              mfma_qk_first(sA[qb], kg[0][0], qf[qb][ks], negm[qb]);
            else
              mfma_qk(sA[qb], kg[ks / GK][ks % GK], qf[qb][ks]);
          }
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) mfma_settle_v(sA[qb]);
        if (win || t_begin * BN + 32 > vis_min) mask_half(sA, 2 * t_begin);
        float mx[QB];
        rowmax_all(sA, mx);
        reference_first(mx, sA);
        if (QB == 2 && t_begin >= t_dead && t_dead < t_end)
          early_events(sA, std::integral_constant<int, QB - 1>{});  // the first step already works on unit 1 alone
        else
          early_events(sA, std::integral_constant<int, 0>{});
        // first K batch of the first step: second half of tile t_begin
#pragma unroll
        for (int j = 0; j < GK; ++j) kg[0][j] = k_frag(j, HALFB);
      }
      int t = t_begin;
      constexpr std::integral_constant<int, 0> both{};
      for (; t < t_lead; ++t) {
        step(sA, sB, 2 * t, std::false_type{}, std::true_type{}, std::true_type{}, both);
        step(sB, sA, 2 * t + 1, std::true_type{}, std::true_type{}, std::true_type{}, both, t + 1 == t_dead && t_dead < t_end);
      }
      for (; t < t_nc; ++t) {
        step(sA, sB, 2 * t, std::false_type{}, std::false_type{}, std::false_type{}, both);
        step(sB, sA, 2 * t + 1, std::true_type{}, std::false_type{}, std::false_type{}, both);
      }
      for (; t < t_fast; ++t) {
        step(sA, sB, 2 * t, std::false_type{}, std::false_type{}, std::true_type{}, both);
        step(sB, sA, 2 * t + 1, std::true_type{}, std::false_type{}, std::true_type{}, both);
      }
      for (; t < t_dead; ++t) {
        step(sA, sB, 2 * t, std::false_type{}, std::true_type{}, std::true_type{}, both);
        step(sB, sA, 2 * t + 1, std::true_type{}, std::true_type{}, std::true_type{}, both, t + 1 == t_dead && t_dead < t_end);
      }
      if constexpr (QB == 2) {
        // unit 0 is done for good (every further key is beyond its last row): unit 1 alone
        constexpr std::integral_constant<int, 1> second{};
        for (; t < t_fast1; ++t) {
          step(sA, sB, 2 * t, std::false_type{}, std::false_type{}, std::true_type{}, second);
          step(sB, sA, 2 * t + 1, std::true_type{}, std::false_type{}, std::true_type{}, second);
        }
        for (; t < t_end; ++t) {
          step(sA, sB, 2 * t, std::false_type{}, std::true_type{}, std::true_type{}, second);
          step(sB, sA, 2 * t + 1, std::true_type{}, std::true_type{}, std::true_type{}, second);
        }
      }
      wait_vm<0>();  // nothing of ours may still be writing LDS when the workgroup retires or starts over
      wait_lds<0>();
      if (!SUM_MODE || exact) break;
      {
        // Did a row sum of any wavefront overflow?  The rings are dead now: their first bytes carry the vote.
        __builtin_amdgcn_s_barrier();
        if (l == 0) *LDS_PTR(int, lds0 + 4u * (unsigned)w) = overflowed;
        __builtin_amdgcn_s_waitcnt(0xC07F);
        __builtin_amdgcn_s_barrier();
        int any_overflow = 0;
#pragma unroll
        for (int ww = 0; ww < 4; ++ww) any_overflow |= *LDS_PTR(const int, lds0 + 4u * (unsigned)ww);
        any_overflow = __builtin_amdgcn_readfirstlane(any_overflow);
        __builtin_amdgcn_s_barrier();  // every wavefront has read the vote before the next pass refills the ring
        if (__builtin_expect(any_overflow == 0, 1)) break;
      }
    }
#pragma unroll
    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
      for (int db = 0; db < DB; ++db) mfma_settle_a(o[qb][db]);
  } else {
    reset_state();
  }

  // ---- epilogue.  O^T leaves through LDS (the rings are dead by now): a lane holds four consecutive
  // columns of one row, which stored directly would be 8- or 16-byte pieces scattered over 32 rows per
  // instruction; turned in LDS, every store instruction writes whole rows, 16 bytes per lane.
  __builtin_amdgcn_s_barrier();  // every wavefront of the workgroup is through with the rings
  const int64_t n_rows = (int64_t)C * Hq;
  constexpr int OROWF = D * 4 + 16;  // padded LDS row: fp32 partials
  constexpr int OROWH = D * 2 + 16;  // padded LDS row: bf16 output
  const unsigned obase = lds0 + (unsigned)(w * kRowsPerUnit * OROWF);  // this wavefront's staging area, reused by its units
#pragma unroll
  for (int qb = 0; qb < QB; ++qb) {
    const float l_tot = pair_sum(l_run[qb]);
    const int tok0 = tok[qb] - m;  // first token of the unit
    if (p.n_splits == 1) {
      const float inv = 1.f / l_tot;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (__bf16)(o[qb][db][rg * 4 + e] * inv);
          *LDS_PTR(bf16x4, obase + (unsigned)(m * OROWH + (db * 32 + 8 * rg + 4 * hi) * 2)) = v;
        }
      if (p.lse && hi == 0 && store_ok[qb])
        p.lse[(int64_t)head[qb] * C + tok[qb]] = (m_run[qb] + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
      constexpr int CPR = D / 8;        // 16-byte chunks per row
      constexpr int RPI = 64 / CPR;     // rows per store instruction
#pragma unroll
      for (int i = 0; i < kRowsPerUnit / RPI; ++i) {
        const int r = i * RPI + l / CPR, c = l % CPR;
        const uintx4 x = *LDS_PTR(const uintx4, obase + (unsigned)(r * OROWH + c * 16));
        if (unit_valid[qb] && tok0 + r < C)
          __builtin_nontemporal_store(x, reinterpret_cast<uintx4*>(reinterpret_cast<__bf16*>(p.out) + ((int64_t)(tok0 + r) * Hq + head[qb]) * D + c * 8));
      }
    } else {
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          floatx4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[qb][db][rg * 4 + e];
          *LDS_PTR(floatx4, obase + (unsigned)(m * OROWF + (db * 32 + 8 * rg + 4 * hi) * 4)) = v;
        }
      if (hi == 0 && store_ok[qb]) {
        float2 ml = make_float2(m_run[qb], l_tot);
        *reinterpret_cast<float2*>(p.part_ml + ((int64_t)split * n_rows + (int64_t)tok[qb] * Hq + head[qb]) * 2) = ml;
      }
      constexpr int CPR = D / 4;        // 16-byte chunks per row
      constexpr int RPI = 64 / CPR;     // rows per store instruction
#pragma unroll
      for (int i = 0; i < kRowsPerUnit / RPI; ++i) {
        const int r = i * RPI + l / CPR, c = l % CPR;
        const floatx4 x = *LDS_PTR(const floatx4, obase + (unsigned)(r * OROWF + c * 16));
        if (unit_valid[qb] && tok0 + r < C)
          __builtin_nontemporal_store(x, reinterpret_cast<floatx4*>(p.part_o + ((int64_t)split * n_rows + (int64_t)(tok0 + r) * Hq + head[qb]) * D + c * 4));
      }
    }
  }
}

template <int D, int QB, int NV>
static hipError_t prepare_one() {
  constexpr int lds_bytes = (2 * NV + 1) * kTileKeys * D * 2;
  // per device: the attribute belongs to the device's copy of the kernel (idempotent; a benign race at worst
  // sets it twice)
  static bool attr_done[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  if (!attr_done[dev]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel<D, QB, NV>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_done[dev] = true;
  }
  return hipSuccess;
}

template <int D, int QB, int NV>
static hipError_t launch_one(const AttnParams& p, hipStream_t s) {
  constexpr int lds_bytes = (2 * NV + 1) * kTileKeys * D * 2;
  hipError_t e = prepare_one<D, QB, NV>();  // a no-op after kvfold_cache_create
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bf16_kernel<D, QB, NV>), dim3(padded_grid(p.n_wgs)), dim3(256), lds_bytes, s, p);
  return hipGetLastError();
}

hipError_t prepare_attn_bf16(int head_dim) {
  hipError_t e = hipErrorInvalidValue;
  if (head_dim == 128) {
    e = prepare_one<128, 2, kRingTwoUnits>();
    if (e == hipSuccess) e = prepare_one<128, 1, kRingOneUnit>();
  } else if (head_dim == 64) {
    e = prepare_one<64, 2, kRingTwoUnits>();
    if (e == hipSuccess) e = prepare_one<64, 1, kRingOneUnit>();
  }
  return e;
}

hipError_t launch_attn_bf16(const AttnParams& p, int head_dim, int qb, hipStream_t s) {
  if (head_dim == 128) return qb == 2 ? launch_one<128, 2, kRingTwoUnits>(p, s) : launch_one<128, 1, kRingOneUnit>(p, s);
  if (head_dim == 64) return qb == 2 ? launch_one<64, 2, kRingTwoUnits>(p, s) : launch_one<64, 1, kRingOneUnit>(p, s);
  return hipErrorInvalidValue;
}

}  // namespace kvfold
