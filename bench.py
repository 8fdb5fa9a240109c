#!/usr/bin/env python3
"""Benchmark of the KV-Fold fold step on one MI355X.

A bench "step" is one complete fold of the headline workload: the Llama-3.1-8B-shaped layer of the
benchmark definition (Hq=32, Hkv=8, d=128, bf16, C=2048, 8 chunks = 16K tokens), i.e. 8 calls of
kvfold_step (append + chunk-prefix attention [+ merge]) starting from an empty cache.  All inputs
are resident in HBM before the timed region.  The headline value is useful attention TFLOP/s
(4*Hq*d*C*(L_prev + (C+1)/2) per fold step, masked pairs not counted) of the whole fold.

One JSON line is printed with the driver's fields plus
  roofline      dominant kernel (chunk-prefix attention) against the bf16 dense MFMA peak, its
                duration measured with HIP events recorded by the library on the step's stream
  cpu_baseline  the fp64 oracle timed on this machine's host cores on a bounded sample of the same
                workload (also used as a spot check of the GPU output)
  extra         tokens/s and TFLOP/s against cache length for this and the long-context shapes
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 MFMA (256 CU x 4096 FLOP/clk x 2.4 GHz)
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM bytes per attention-kernel launch (mean over the launches of one fold), from two rocprofv3 --pmc
# runs of this script (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch), each scaled by what the same
# counter reads for the append kernel, a plain copy of known size (write factor 1.000, fetch factor
# 1.99; summaries under profiles/).  Keyed by (workload, tuning); other combinations report null.
MEASURED_HBM_TRAFFIC_BYTES = {("llama_16k", ()): 88.1e6, ("full_stack_128k", ()): 637e6,
                              ("llama_16k", ((3, 1),)): 71.6e6, ("full_stack_128k", ((3, 1),)): 611e6}


def step_flops(cfg, C, L_prev):
    """Useful FLOPs of one fold step: QK^T and PV over the unmasked (row, key) pairs."""
    return 4.0 * cfg.n_q_heads * cfg.head_dim * C * (L_prev + (C + 1) / 2.0)


def step_bytes(cfg, C, L_prev):
    """Algorithmic HBM bytes of one fold step: cache read once, q read, out written, append read+write."""
    es = 2 if cfg.dtype == "bf16" else 4
    L = L_prev + C
    return (2 * cfg.n_kv_heads * cfg.head_dim * L * es + 2 * C * cfg.n_q_heads * cfg.head_dim * es
            + 4 * C * cfg.n_kv_heads * cfg.head_dim * es)


class Workload:
    """All chunks of one layer resident on the GPU + a library cache."""

    def __init__(self, cfg, torch, kv, I, device, n_steps=None, tuning=None, rope=False):
        self.cfg, self.torch = cfg, torch
        self.n_steps = n_steps or cfg.n_steps
        self.cache = kv.KvFoldCache(1, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.chunk,
                                    self.n_steps * cfg.chunk, cfg.dtype, device=device.index or 0)
        for knob, val in (tuning or {}).items():
            self.cache.set_tuning(knob, val)
        self.chunks = [I.chunk_qkv(cfg, 0, s, device=device) for s in range(self.n_steps)]
        self.out = torch.empty_like(self.chunks[0][0])
        # rope: the step rotates q and k_new itself at the chunk's absolute positions (kvfold_step_rope)
        self.rope = [I.rope_tables(cfg.head_dim, s * cfg.chunk, cfg.chunk, device=device) for s in range(self.n_steps)] \
            if rope else [None] * self.n_steps
        self.flops = sum(step_flops(cfg, cfg.chunk, s * cfg.chunk) for s in range(self.n_steps))
        self.bytes = sum(step_bytes(cfg, cfg.chunk, s * cfg.chunk) for s in range(self.n_steps))

    def fold(self):
        self.cache.set_length(0, 0)
        for s, (q, k, v) in enumerate(self.chunks):
            self.cache.step(0, q, k, v, self.out, pos_offset=s * self.cfg.chunk, rope=self.rope[s])

    def per_step_curve(self, reps=3):
        """Event-timed single steps against a cache rewound to each length: [(L_prev, ms)]."""
        torch = self.torch
        self.fold()
        torch.cuda.synchronize()
        res = []
        for s, (q, k, v) in enumerate(self.chunks):
            best = None
            for _ in range(reps):
                self.cache.set_length(0, s * self.cfg.chunk)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                self.cache.step(0, q, k, v, self.out, pos_offset=s * self.cfg.chunk)
                e1.record()
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            res.append((s * self.cfg.chunk, best))
        return res

    def close(self):
        self.cache.close()


def time_folds(w, torch, steps, warmup):
    for _ in range(warmup):
        w.fold()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        w.fold()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def profiled_folds(w, steps):
    """Same folds with the library's per-kernel HIP events: returns summed kernel milliseconds."""
    w.cache.profile_begin(steps * w.n_steps)
    for _ in range(steps):
        w.fold()
    n, append_ms, attn_ms, merge_ms = w.cache.profile_end()
    return n, append_ms, attn_ms, merge_ms


def cpu_baseline(w, torch):
    """Time the fp64 oracle, as it stands, on the last two fold steps of the workload (all rows, all
    heads: about 1 TFLOP of fp64 for the headline workload, 10-20 s on 16 host cores) and compare the
    GPU output of the last step with it."""
    import numpy as np
    from oracle import kvfold_oracle as O
    cfg = w.cfg
    O.build()
    store = np.uint16 if cfg.dtype == "bf16" else np.float32

    def bits(t):
        t = t.cpu().contiguous()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    n_timed = min(2, w.n_steps)
    oc = O.OracleCache(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, w.n_steps * cfg.chunk, store_dtype=store)
    for q, k, v in w.chunks[:-n_timed]:
        oc.append(bits(k), bits(v))
    host = [(q.cpu().double().numpy(), bits(k), bits(v)) for q, k, v in w.chunks[-n_timed:]]
    flops, tokens, ref = 0.0, 0, None
    t0 = time.perf_counter()
    for q, k, v in host:
        flops += step_flops(cfg, cfg.chunk, oc.len)
        tokens += cfg.chunk
        ref, _ = oc.step(q, k, v, oc.len)
    dt = time.perf_counter() - t0
    # GPU output of the last step
    w.fold()
    torch.cuda.synchronize()
    err = float(np.abs(w.out.cpu().double().numpy() - ref).max())
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": O.threads(), "kind": "oracle",
        "sample": f"last {n_timed} fold steps of the workload (C={cfg.chunk}, cache length up to {oc.len}), every row and head: "
                  f"{flops / 1e9:.0f} GFLOP fp64 in {dt:.1f} s",
        "fold_tokens_per_s": tokens / dt, "gpu_max_abs_err_vs_oracle_last_step": err,
    }


def decode_shaped_points(torch, kv, I, dev, L=131072, chunks=(1, 4, 16), reps=20):
    """Fold steps of 1..16 tokens against a 128K cache of the Llama-shaped layer (the greedy decode
    that follows the chain in the needle protocol, Sec. 4): HBM-bound, reported against the 8 TB/s
    peak.  The cache rows are seeded N(0,1) written in place; each step is timed with the library's
    HIP events (append, attention, merge) over `reps` repeats against the rewound cache."""
    cfg = I.CONFIGS["llama_16k"]
    pts = []
    for C in chunks:
        Lp = L - C
        cache = kv.KvFoldCache(1, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, C, L, "bf16", device=dev.index or 0)
        g = torch.Generator(device=dev)
        g.manual_seed(I.BASE_SEED + C)
        K, V = cache.view(0)
        K.normal_(generator=g)
        V.normal_(generator=g)
        q, k, v = (torch.randn((C, h, cfg.head_dim), device=dev, generator=g).bfloat16()
                   for h in (cfg.n_q_heads, cfg.n_kv_heads, cfg.n_kv_heads))
        out = torch.empty_like(q)
        for _ in range(3):
            cache.set_length(0, Lp)
            cache.step(0, q, k, v, out, pos_offset=Lp)
        torch.cuda.synchronize()
        cache.profile_begin(reps)
        t0 = time.perf_counter()
        for _ in range(reps):
            cache.set_length(0, Lp)
            cache.step(0, q, k, v, out, pos_offset=Lp)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / reps
        n, a_ms, t_ms, m_ms = cache.profile_end()
        nbytes = step_bytes(cfg, C, Lp)
        pts.append({
            "C": C, "L_prev": Lp, "plan_workgroups_splits": list(cache.plan(C, L)),
            "step_ms": wall_ms, "append_ms": a_ms / n, "attention_ms": t_ms / n, "merge_ms": m_ms / n,
            "tokens_per_s": C / (wall_ms * 1e-3), "algorithmic_bytes": nbytes,
            "roofline": {"kernel": "attn_bf16_kernel", "bound": "hbm", "achieved": nbytes / (t_ms / n * 1e-3) / 1e9,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": nbytes / (t_ms / n * 1e-3) / 1e9 / PEAK_HBM_GBS},
            "step_GBps": nbytes / (wall_ms * 1e-3) / 1e9,
        })
        cache.close()
    return pts


def box_peaks(torch, dev):
    """What this machine delivers on plain library work, measured in the same run, to put the datasheet fractions
    beside measured ones: a large bf16 GEMM (torch.matmul, 8192^3), a read-only pass over 2 GiB (sum) and a
    1 GiB copy.  Best of a few repeats each."""
    def best_ms(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        b = None
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            b = ms if b is None else min(b, ms)
        return b
    n = 8192
    g = torch.Generator(device=dev)
    g.manual_seed(1)
    a = torch.randn((n, n), device=dev, generator=g).bfloat16()
    b = torch.randn((n, n), device=dev, generator=g).bfloat16()
    gemm_ms = best_ms(lambda: torch.matmul(a, b))
    del a, b
    x = torch.empty(1 << 29, dtype=torch.float32, device=dev).normal_(generator=g)   # 2 GiB
    read_ms = best_ms(lambda: x.sum())
    y = torch.empty(1 << 28, dtype=torch.float32, device=dev)                         # 1 GiB
    copy_ms = best_ms(lambda: y.copy_(x[: 1 << 28]))
    del x, y
    torch.cuda.empty_cache()
    return {"bf16_gemm_8192_tflops": 2.0 * n ** 3 / (gemm_ms * 1e-3) / 1e12,
            "hbm_read_GBps": (1 << 31) / (read_ms * 1e-3) / 1e9,
            "hbm_copy_GBps_read_plus_write": 2.0 * (1 << 30) / (copy_ms * 1e-3) / 1e9}


def fp32_last_step(torch, kv, I, dev, reps=3):
    """The fp32 correctness mode on the last step of the sweep workload at C=2048 (Hq=28, Hkv=4, d=128, 62K-key
    prefix), against the fp32 MFMA peak.  The prefix rows are seeded N(0,1) written in place."""
    cfg = I.CONFIGS["sweep_64k"]
    C, L = 2048, cfg.total_tokens
    Lp = L - C
    cache = kv.KvFoldCache(1, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, C, L, "f32", device=dev.index or 0)
    g = torch.Generator(device=dev)
    g.manual_seed(I.BASE_SEED + 77)
    K, V = cache.view(0)
    K.normal_(generator=g)
    V.normal_(generator=g)
    q, k, v = (torch.randn((C, h, cfg.head_dim), device=dev, generator=g)
               for h in (cfg.n_q_heads, cfg.n_kv_heads, cfg.n_kv_heads))
    out = torch.empty_like(q)
    best = None
    for _ in range(reps):
        cache.set_length(0, Lp)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        cache.step(0, q, k, v, out, pos_offset=Lp)
        e1.record()
        e1.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    cache.close()
    fl = step_flops(cfg.with_(dtype="f32"), C, Lp)
    return {"C": C, "L_prev": Lp, "ms": best, "tflops": fl / (best * 1e-3) / 1e12,
            "frac_of_fp32_mfma_peak": fl / (best * 1e-3) / 1e12 / PEAK_FP32_TFLOPS}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama_16k")
    ap.add_argument("--no-extra", action="store_true", help="skip the long-context curves")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--units-per-wave", type=int, default=0)
    ap.add_argument("--decode-shaped-only", action="store_true",
                    help="run only the decode-shaped points (1..16 tokens against a 128K cache) and print them: for profiling")
    ap.add_argument("--separate-append", action="store_true",
                    help="run the append as its own kernel (a plain copy of known size: the calibration of the HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2605_12471_amd as kv
    from paper_2605_12471_amd import inputs as I

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    kv.load_library()  # fails loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.decode_shaped_only:
        print(json.dumps({"decode_shaped_128k": decode_shaped_points(torch, kv, I, dev)}))
        return
    cfg = I.CONFIGS[args.workload]
    tuning = {}
    if args.splits:
        tuning[kv.TUNE_SPLITS] = args.splits
    if args.units_per_wave:
        tuning[kv.TUNE_UNITS_PER_WAVE] = args.units_per_wave
    if args.separate_append:
        tuning[kv.TUNE_FUSED_APPEND] = 1

    w = Workload(cfg, torch, kv, I, dev, tuning=tuning)
    ms = time_folds(w, torch, args.steps, args.warmup)
    tflops = w.flops / (ms * 1e-3) / 1e12
    tokens_per_s = cfg.total_tokens / (ms * 1e-3)

    n_prof, append_ms, attn_ms, merge_ms = profiled_folds(w, args.steps)
    attn_avg_ms = attn_ms / max(n_prof, 1)
    attn_tflops = (w.flops * args.steps) / (attn_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    roofline = {
        "kernel": "attn_bf16_kernel" if cfg.dtype == "bf16" else "attn_f32_kernel",
        "bound": "mfma", "achieved": attn_tflops, "peak": peak, "unit": "TFLOP/s", "frac": attn_tflops / peak,
        "traffic": MEASURED_HBM_TRAFFIC_BYTES.get((cfg.name, tuple(sorted(tuning.items())))),
        "launches": n_prof, "avg_launch_ms": attn_avg_ms, "flops_per_launch_avg": w.flops / w.n_steps,
        "algorithmic_bytes_per_launch_avg": w.bytes / w.n_steps,
        "achieved_hbm_GBps_algorithmic": w.bytes * args.steps / (attn_ms * 1e-3) / 1e9,
        "append_ms_avg": append_ms / max(n_prof, 1), "merge_ms_avg": merge_ms / max(n_prof, 1),
    }

    extra = {}
    curve = w.per_step_curve()
    extra["curve_" + cfg.name] = [
        {"L_prev": L, "ms": t, "tflops": step_flops(cfg, cfg.chunk, L) / (t * 1e-3) / 1e12,
         "tokens_per_s": cfg.chunk / (t * 1e-3)} for L, t in curve]

    result = {
        "metric": "chunk-prefix attention TFLOP/s (useful FLOPs of a whole fold / wall time)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: 1 layer, Hq={cfg.n_q_heads}, Hkv={cfg.n_kv_heads}, d={cfg.head_dim}, "
                               f"C={cfg.chunk}, fold to {cfg.total_tokens} tokens ({cfg.n_steps} steps)",
                   "seed": I.BASE_SEED, "step": "one whole fold from an empty cache"},
        "frac_of_bf16_peak": tflops / PEAK_BF16_TFLOPS, "fold_tokens_per_s": tokens_per_s,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, torch)
    w.close()

    if not args.no_extra:
        # long-context operating points of the benchmark definition (single layer each)
        for name, n_steps in (("full_stack_128k", None), ("deep_chain_128k", None), ("sweep_64k", None)):
            c2 = I.CONFIGS[name].with_(n_layers=1)
            w2 = Workload(c2, torch, kv, I, dev, tuning=tuning)
            w2.fold()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            w2.fold()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            n, a_ms, t_ms, m_ms = profiled_folds(w2, 1)
            pts = w2.per_step_curve(reps=2)
            sel = pts if len(pts) <= 32 else pts[:: len(pts) // 16] + [pts[-1]]
            extra["fold_" + name] = {
                "workload": f"Hq={c2.n_q_heads}, Hkv={c2.n_kv_heads}, d={c2.head_dim}, C={c2.chunk}, "
                            f"{c2.total_tokens} tokens, 1 layer",
                "fold_ms": dt * 1e3, "tflops": w2.flops / dt / 1e12, "frac_of_bf16_peak": w2.flops / dt / 1e12 / PEAK_BF16_TFLOPS,
                "tokens_per_s": c2.total_tokens / dt,
                "attention_kernel_tflops": w2.flops / (t_ms * 1e-3) / 1e12,
                "attention_ms": t_ms, "append_ms": a_ms, "merge_ms": m_ms,
                "algorithmic_GBps": w2.bytes / dt / 1e9,
                "curve": [{"L_prev": L, "ms": t, "tflops": step_flops(c2, c2.chunk, L) / (t * 1e-3) / 1e12,
                           "tokens_per_s": c2.chunk / (t * 1e-3),
                           "algorithmic_GBps": step_bytes(c2, c2.chunk, L) / (t * 1e-3) / 1e9} for L, t in sel],
            }
            w2.close()
        # config 5: the same 64K tokens folded with every chunk size of the sweep (bf16)
        sweep = []
        for C in (128, 512, 2048, 8192):
            c5 = I.CONFIGS["sweep_64k"].with_(chunk=C)
            w5 = Workload(c5, torch, kv, I, dev, tuning=tuning)
            w5.fold()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            w5.fold()
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            sweep.append({"C": C, "steps": c5.n_steps, "plan_last_step_workgroups_splits": list(w5.cache.plan(C, c5.total_tokens)),
                          "fold_ms": dt * 1e3, "tflops": w5.flops / dt / 1e12,
                          "frac_of_bf16_peak": w5.flops / dt / 1e12 / PEAK_BF16_TFLOPS, "tokens_per_s": c5.total_tokens / dt})
            w5.close()
        extra["chunk_size_sweep_64k"] = sweep
        extra["decode_shaped_128k"] = decode_shaped_points(torch, kv, I, dev)
        extra["fp32_mode_sweep_64k_last_step"] = fp32_last_step(torch, kv, I, dev)
        extra["box_peaks_measured"] = box_peaks(torch, dev)
        # the headline fold with unrotated inputs: rotary embedding applied inside the step
        w3 = Workload(cfg, torch, kv, I, dev, tuning=tuning, rope=True)
        ms3 = time_folds(w3, torch, args.steps, args.warmup)
        extra["fold_" + cfg.name + "_rope_in_step"] = {
            "ms_per_fold": ms3, "tflops": w3.flops / (ms3 * 1e-3) / 1e12, "ms_per_fold_without": ms,
            "note": "same workload through kvfold_step_rope (q, k_new unrotated; cos/sin tables resident)"}
        w3.close()
        # ... and with the carried cache round-tripped through int8 at every step (storage perturbation, Sec. 8)
        w4 = Workload(cfg, torch, kv, I, dev, tuning=tuning)
        w4.cache.set_storage_roundtrip(8)
        ms4 = time_folds(w4, torch, args.steps, args.warmup)
        extra["fold_" + cfg.name + "_int8_roundtrip"] = {
            "ms_per_fold": ms4, "tflops": w4.flops / (ms4 * 1e-3) / 1e12, "ms_per_fold_without": ms,
            "note": "rows quantised in place (per-row absmax, bf16 -> int8 -> bf16) by their own kernel after a separate append"}
        w4.close()
    result["extra"] = extra
    print(json.dumps(result))


if __name__ == "__main__":
    main()
