#!/usr/bin/env python3
"""Benchmark of the KV-Fold fold step on one MI355X.

A bench "step" is one complete fold of the headline workload, the largest single-GPU configuration of the
benchmark definition: 32 independent Llama-3.1-8B-shaped layers (Hq=32, Hkv=8, d=128, bf16), chunks of C=4096
tokens folded to 128K tokens -- 32 chunks x 32 layers = 1024 calls of kvfold_step (append + chunk-prefix
attention) from an empty cache, chunk by chunk through all layers as a model would, with the 16 GiB of K/V of
the paper's Tab. 4 accounting resident in HBM.  Every input chunk of every layer (51 GB) is resident in HBM
before the timed region.  The headline value is useful attention TFLOP/s of the whole fold
(4*Hq*d*C*(L_prev + (C+1)/2) per fold step, masked pairs not counted): 4.50 PFLOP per bench step.

One compact JSON line is printed with the driver's fields plus
  roofline      dominant kernel (chunk-prefix attention) against the bf16 dense MFMA peak; its duration comes
                from HIP events that the library records on the step's stream around every launch of the
                timed region itself
  cpu_baseline  the fp64 oracle timed on this machine's host cores on a bounded sample of the same workload
                (also used as a spot check of the GPU output)
  curve         TFLOP/s and tokens/s of single steps against the cache length (one layer of the workload)
  extra         one-line summaries of the other workloads of the benchmark definition (16K fold, depth-511
                chain at C=256, chunk-size sweep, decode-shaped steps, fp32 mode, sink+window steps)
`--detail PATH` also writes every per-step curve as JSON to PATH.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # MI355X dense bf16 MFMA (256 CU x 4096 FLOP/clk x 2.4 GHz)
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

KERNEL_SOURCES = ("attn_bf16.hip", "kvfold_internal.h", "kvfold_consts.h")


def kernel_source_hash():
    """Short hash of the attention kernel's code -- its sources with comments and white space taken out: a measured
    HBM-traffic figure is only reported for the kernel it was measured on, and rewording a comment does not make
    it another kernel."""
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2605_12471_amd", "csrc", name), "r") as f:
            text = f.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)     # block comments
        text = re.sub(r"//[^\n]*", "", text)                   # line comments (no string in these files holds //)
        h.update("".join(text.split()).encode())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """HBM bytes per attention launch from the committed rocprofv3 counter summary of this workload
    (profiles/attn_bf16_<workload>.md, line `traffic_bytes_per_launch: <bytes> kernel_source: <hash>`),
    or None when there is none for the kernel sources as they are now."""
    path = os.path.join(ROOT, "profiles", f"attn_bf16_{workload}.md")
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)\s+kernel_source:\s*([0-9a-f]+)", text)
    if not m or m.group(2) != kernel_source_hash():
        return None
    return float(m.group(1))


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
    """All chunks of all layers resident on the GPU + a library cache."""

    def __init__(self, cfg, torch, kv, I, device, n_steps=None, tuning=None, rope=False, storage_bits=0):
        self.cfg, self.torch = cfg, torch
        self.n_steps = n_steps or cfg.n_steps
        self.n_layers = cfg.n_layers
        self.cache = kv.KvFoldCache(cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.chunk,
                                    self.n_steps * cfg.chunk, cfg.dtype, device=device.index or 0)
        for knob, val in (tuning or {}).items():
            self.cache.set_tuning(knob, val)
        if storage_bits:
            self.cache.set_storage_roundtrip(storage_bits)
        # chunks[step][layer] = (q, k_new, v_new)
        self.chunks = [[I.chunk_qkv(cfg, l, s, device=device) for l in range(cfg.n_layers)] for s in range(self.n_steps)]
        self.out = torch.empty_like(self.chunks[0][0][0])
        # rope: the step rotates q and k_new itself at the chunk's absolute positions (kvfold_step_rope)
        self.rope = [I.rope_tables(cfg.head_dim, s * cfg.chunk, cfg.chunk, device=device) for s in range(self.n_steps)] \
            if rope else [None] * self.n_steps
        per_layer = sum(step_flops(cfg, cfg.chunk, s * cfg.chunk) for s in range(self.n_steps))
        self.flops = per_layer * cfg.n_layers
        self.bytes = sum(step_bytes(cfg, cfg.chunk, s * cfg.chunk) for s in range(self.n_steps)) * cfg.n_layers
        self.launches = self.n_steps * cfg.n_layers

    def fold(self):
        """Chunk by chunk through all layers, from an empty cache."""
        self.cache.set_length(-1, 0)
        for s, per_layer in enumerate(self.chunks):
            for l, (q, k, v) in enumerate(per_layer):
                self.cache.step(l, q, k, v, self.out, pos_offset=s * self.cfg.chunk, rope=self.rope[s])

    def per_step_curve(self, reps=3, layer=0):
        """Event-timed single steps of one layer against a cache rewound to each length: [(L_prev, ms)]."""
        torch = self.torch
        self.fold()
        torch.cuda.synchronize()
        res = []
        for s, per_layer in enumerate(self.chunks):
            q, k, v = per_layer[layer]
            best = None
            for _ in range(reps):
                self.cache.set_length(layer, s * self.cfg.chunk)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                self.cache.step(layer, q, k, v, self.out, pos_offset=s * self.cfg.chunk)
                e1.record()
                e1.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            res.append((s * self.cfg.chunk, best))
        return res

    def close(self):
        self.cache.close()


def time_folds(w, torch, steps, warmup, events=False):
    """Wall time per fold over `steps` folds after `warmup` untimed ones; with events=True the library
    records HIP events around every kernel of the timed folds: returns (ms, (n, append, attn, merge) | None)."""
    for _ in range(warmup):
        w.fold()
    torch.cuda.synchronize()
    if events:
        w.cache.profile_begin(steps * w.launches)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        w.fold()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    return ms, (w.cache.profile_end() if events else None)


def cpu_baseline(w, torch, I, n_rows, layer=0):
    """Time the fp64 oracle, as it stands, on seeded sample rows (all heads) of the last fold step of one layer
    of the workload, and compare the GPU output of that step with it."""
    import numpy as np
    from oracle import kvfold_oracle as O
    cfg = w.cfg
    O.build()
    store = np.uint16 if cfg.dtype == "bf16" else np.float32

    def bits(t):
        t = t.cpu().contiguous()
        return t.view(torch.int16).numpy().view(np.uint16) if t.dtype == torch.bfloat16 else t.numpy()

    last = w.n_steps - 1
    oc = O.OracleCache(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, w.n_steps * cfg.chunk, store_dtype=store)
    for s in range(last):
        _, k, v = w.chunks[s][layer]
        oc.append(bits(k), bits(v))
    q, k, v = w.chunks[last][layer]
    rows = I.sample_rows(cfg, last, n_random=max(n_rows - 5, 0))
    qh, kh, vh = q.cpu().double().numpy(), bits(k), bits(v)
    L_prev = oc.len
    oc.append(kh, vh)
    flops = sum(4.0 * cfg.n_q_heads * cfg.head_dim * (L_prev + r + 1) for r in rows)
    t0 = time.perf_counter()
    ref, _ = oc.attend(qh, L_prev, rows=rows)
    dt = time.perf_counter() - t0
    # GPU output of the same step: rewind that layer by one chunk and redo it
    w.cache.set_length(layer, L_prev)
    w.cache.step(layer, q, k, v, w.out, pos_offset=L_prev)
    torch.cuda.synchronize()
    err = float(np.abs(w.out[rows].cpu().double().numpy() - ref).max())
    return {
        "value": round(flops / dt / 1e12, 5), "unit": "TFLOP/s", "cores": O.threads(), "kind": "oracle",
        "sample": f"{len(rows)} seeded rows x {cfg.n_q_heads} heads of layer {layer}'s last step "
                  f"({L_prev + cfg.chunk} keys): {flops / 1e9:.0f} GFLOP fp64 in {dt:.1f} s",
        "gpu_max_abs_err_on_sample": round(err, 6),
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


def window_steps(torch, kv, I, dev, L=131072, C=256, n_sink=4, window=1020, reps=200):
    """Steps of the paper's deep chain (C = 256 at 128K tokens) under the streaming baseline's mask, 4 sink tokens +
    1020 recent tokens (Sec. 6), through kvfold_step_window: work and bytes follow the window, not the cache.
    `reps` steps back to back against the rewound cache, wall-clock per step; the plain step beside it."""
    cfg = I.CONFIGS["deep_chain_128k"]
    Lp = L - C
    cache = kv.KvFoldCache(1, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, C, L, "bf16", device=dev.index or 0)
    g = torch.Generator(device=dev)
    g.manual_seed(I.BASE_SEED + 4)
    K, V = cache.view(0)
    K.normal_(generator=g)
    V.normal_(generator=g)
    q, k, v = (torch.randn((C, h, cfg.head_dim), device=dev, generator=g).bfloat16()
               for h in (cfg.n_q_heads, cfg.n_kv_heads, cfg.n_kv_heads))
    out = torch.empty_like(q)
    res = {}
    for name, win in (("window", (n_sink, window)), ("plain", None)):
        for timed in (False, True):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps if timed else 5):
                cache.set_length(0, Lp)
                cache.step(0, q, k, v, out, pos_offset=Lp, window=win)
            torch.cuda.synchronize()
            res[name] = (time.perf_counter() - t0) / reps
    cache.close()
    es, Hq, Hkv, d = 2, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    keys = n_sink + window                                   # keys per row
    rows_kv = n_sink + window + C - 1                        # distinct cache rows the chunk's rows see
    flops = 4.0 * Hq * d * C * keys
    nbytes = 2 * Hkv * d * es * rows_kv + 2 * C * Hq * d * es + 4 * C * Hkv * d * es
    t = res["window"]
    return {"C": C, "L_prev": Lp, "n_sink": n_sink, "window": window, "step_us": t * 1e6, "plain_step_us": res["plain"] * 1e6,
            "flops": flops, "algorithmic_bytes": nbytes, "tflops": flops / t / 1e12, "algorithmic_GBps": nbytes / t / 1e9,
            "tokens_per_s": C / t}


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


def curve_points(cfg, pts):
    return [{"L_prev": L, "ms": t, "tflops": step_flops(cfg, cfg.chunk, L) / (t * 1e-3) / 1e12,
             "tokens_per_s": cfg.chunk / (t * 1e-3), "algorithmic_GBps": step_bytes(cfg, cfg.chunk, L) / (t * 1e-3) / 1e9}
            for L, t in pts]


def single_layer_fold(name, torch, kv, I, dev, tuning, chunk=None, reps=3, curve=True, **wkw):
    """One layer of a workload of the benchmark definition: best wall time of `reps` folds, the library's
    per-kernel event times of one more fold, and (optionally) the per-step curve."""
    c = I.CONFIGS[name].with_(n_layers=1)
    if chunk:
        c = c.with_(chunk=chunk)
    w = Workload(c, torch, kv, I, dev, tuning=tuning, **wkw)
    w.fold()
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        t0 = time.perf_counter()
        w.fold()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        best = dt if best is None else min(best, dt)
    _, (n, a_ms, t_ms, m_ms) = time_folds(w, torch, 1, 0, events=True)
    d = {"workload": f"Hq={c.n_q_heads}, Hkv={c.n_kv_heads}, d={c.head_dim}, C={c.chunk}, {c.total_tokens} tokens, 1 layer",
         "plan_last_step_workgroups_splits": list(w.cache.plan(c.chunk, c.total_tokens)),
         "fold_ms": best * 1e3, "tflops": w.flops / best / 1e12, "frac_of_bf16_peak": w.flops / best / 1e12 / PEAK_BF16_TFLOPS,
         "tokens_per_s": c.total_tokens / best, "attention_kernel_tflops": w.flops / (t_ms * 1e-3) / 1e12,
         "attention_ms": t_ms, "append_ms": a_ms, "merge_ms": m_ms, "algorithmic_GBps": w.bytes / best / 1e9}
    if curve:
        pts = w.per_step_curve(reps=2)
        d["curve"] = curve_points(c, pts if len(pts) <= 32 else pts[:: len(pts) // 16] + [pts[-1]])
    w.close()
    return d


def r(x, n=1):
    return round(float(x), n)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="full_stack_128k")
    ap.add_argument("--layers", type=int, default=0, help="override the workload's number of layers (0 = as defined)")
    ap.add_argument("--chunk", type=int, default=0, help="override the workload's chunk length (0 = as defined)")
    ap.add_argument("--dtype", default="", choices=["", "bf16", "f32"], help="override the workload's element type")
    ap.add_argument("--no-extra", action="store_true", help="skip the other workloads")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-rows", type=int, default=400, help="sample rows of the oracle's timed leg")
    ap.add_argument("--detail", default="", help="write per-step curves of every workload to this JSON file")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--units-per-wave", type=int, default=0)
    ap.add_argument("--decode-shaped-only", action="store_true",
                    help="run only the decode-shaped points (1..16 tokens against a 128K cache) and print them: for profiling")
    ap.add_argument("--window-only", action="store_true",
                    help="run only the sink + sliding-window steps (4 + 1020 at C = 256 against 128K) and print them: for profiling")
    ap.add_argument("--peaks-only", action="store_true",
                    help="run only kvfold_measure_peaks (bf16 matrix instructions alone, streaming HBM read) and print it")
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
    if args.peaks_only:
        rc, box_tflops, box_gbps = kv.kvfold_measure_peaks(0)
        if rc:
            raise kv.KvFoldError(rc, "kvfold_measure_peaks")
        print(json.dumps({"box_peaks": {"mfma_only_bf16_tflops": box_tflops, "hbm_read_GBps": box_gbps}}))
        return
    if args.decode_shaped_only:
        print(json.dumps({"decode_shaped_128k": decode_shaped_points(torch, kv, I, dev)}))
        return
    if args.window_only:
        print(json.dumps({"window_4_1020_C256_128k": window_steps(torch, kv, I, dev)}))
        return
    cfg = I.CONFIGS[args.workload]
    if args.layers:
        cfg = cfg.with_(n_layers=args.layers)
    if args.chunk:
        cfg = cfg.with_(chunk=args.chunk)
    if args.dtype:
        cfg = cfg.with_(dtype=args.dtype)
    tuning = {}
    if args.splits:
        tuning[kv.TUNE_SPLITS] = args.splits
    if args.units_per_wave:
        tuning[kv.TUNE_UNITS_PER_WAVE] = args.units_per_wave
    if args.separate_append:
        tuning[kv.TUNE_FUSED_APPEND] = 1

    t_setup = time.perf_counter()
    w = Workload(cfg, torch, kv, I, dev, tuning=tuning)
    torch.cuda.synchronize()
    print(f"bench: {cfg.name} inputs resident ({torch.cuda.memory_allocated() / 2**30:.1f} GiB allocated by torch, "
          f"{w.cache.cfg.n_layers} layers) after {time.perf_counter() - t_setup:.1f} s", file=sys.stderr, flush=True)
    ms, (n_prof, append_ms, attn_ms, merge_ms) = time_folds(w, torch, args.steps, args.warmup, events=True)
    print(f"bench: timed region done, {ms:.1f} ms per fold", file=sys.stderr, flush=True)
    tflops = w.flops / (ms * 1e-3) / 1e12
    tokens_per_s = cfg.total_tokens / (ms * 1e-3)

    attn_avg_ms = attn_ms / max(n_prof, 1)
    attn_tflops = (w.flops * args.steps) / (attn_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if cfg.dtype == "bf16" else PEAK_FP32_TFLOPS
    roofline = {
        "kernel": "attn_bf16_kernel" if cfg.dtype == "bf16" else "attn_f32_kernel",
        "bound": "mfma", "achieved": r(attn_tflops), "peak": peak, "unit": "TFLOP/s", "frac": r(attn_tflops / peak, 4),
        "traffic": None if tuning or args.dtype or args.layers else measured_traffic(cfg.name + (f"_C{args.chunk}" if args.chunk else "")),
        "launches": n_prof, "avg_launch_ms": r(attn_avg_ms, 4), "flops_per_launch": round(w.flops / w.launches),
        "algorithmic_bytes_per_launch": round(w.bytes / w.launches),
    }
    detail_roofline = dict(roofline, append_ms_avg=append_ms / max(n_prof, 1), merge_ms_avg=merge_ms / max(n_prof, 1),
                           kernel_source=kernel_source_hash())

    detail = {}
    pts = curve_points(cfg, w.per_step_curve(reps=2))
    detail["curve_" + cfg.name] = pts
    sel = pts if len(pts) <= 8 else pts[:: len(pts) // 4] + [pts[-1]]
    curve = {"what": "layer-0 steps vs length before the step",
             "L_prev": [p["L_prev"] for p in sel], "tflops": [round(p["tflops"]) for p in sel],
             "tokens_per_s": [round(p["tokens_per_s"]) for p in sel]}

    result = {
        "metric": "chunk-prefix attention TFLOP/s of a whole fold (useful FLOPs / wall time)",
        "value": r(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.n_layers} layers, Hq={cfg.n_q_heads}, Hkv={cfg.n_kv_heads}, d={cfg.head_dim}, "
                               f"C={cfg.chunk}, fold to {cfg.total_tokens} tokens = {w.launches} kvfold_step calls per bench "
                               f"step ({w.flops / 1e15:.3g} PFLOP), {w.cache.bytes_required() / 2**30:.3g} GiB of K/V resident",
                   "seed": I.BASE_SEED},
        "frac_of_bf16_peak": r(tflops / PEAK_BF16_TFLOPS, 4), "fold_tokens_per_s": round(tokens_per_s),
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        print("bench: oracle leg", file=sys.stderr, flush=True)
        result["cpu_baseline"] = cpu_baseline(w, torch, I, args.cpu_rows)
    w.close()
    del w
    torch.cuda.empty_cache()
    result["curve"] = curve

    if not args.no_extra:
        extra = {}
        # what this machine delivers right after the headline fold: a loop of nothing but bf16 matrix instructions, and a
        # plain streaming read of 2 GiB (both in the library, kvfold_measure_peaks)
        rc, box_tflops, box_gbps = kv.kvfold_measure_peaks(dev.index or 0)
        if rc:
            raise kv.KvFoldError(rc, "kvfold_measure_peaks")
        extra["box_peaks"] = {"mfma_only_tflops": round(box_tflops), "hbm_read_GBps": round(box_gbps),
                              "headline_vs_mfma_only": r(tflops / box_tflops, 3)}
        detail["box_peaks"] = {"mfma_only_bf16_tflops": box_tflops, "hbm_read_GBps": box_gbps}
        # the other workloads of the benchmark definition, one layer each
        for name in ("llama_16k", "deep_chain_128k"):
            print("bench: extra", name, file=sys.stderr, flush=True)
            d = single_layer_fold(name, torch, kv, I, dev, tuning, reps=5 if name == "llama_16k" else 2)
            detail["fold_" + name] = d
            extra[name] = {"tflops": round(d["tflops"]), "frac": r(d["frac_of_bf16_peak"], 3),
                           "attn_tflops": round(d["attention_kernel_tflops"]), "fold_ms": r(d["fold_ms"], 2),
                           "merge_ms": r(d["merge_ms"], 2),
                           "step_tflops_first_last": [round(d["curve"][0]["tflops"]), round(d["curve"][-1]["tflops"])]}
        # config 5: the same 64K tokens folded with every chunk size of the sweep (bf16)
        sweep = {}
        for C in (128, 512, 2048, 8192):
            print("bench: extra sweep_64k C =", C, file=sys.stderr, flush=True)
            d = single_layer_fold("sweep_64k", torch, kv, I, dev, tuning, chunk=C, reps=2, curve=(C == 2048))
            detail[f"fold_sweep_64k_C{C}"] = d
            sweep[f"C{C}"] = [round(d["tflops"]), r(d["frac_of_bf16_peak"], 3)]
        sweep["what"] = "[TFLOP/s, frac of peak]"
        extra["sweep_64k"] = sweep
        print("bench: extra decode", file=sys.stderr, flush=True)
        dec = decode_shaped_points(torch, kv, I, dev)
        detail["decode_shaped_128k"] = dec
        extra["decode_128k"] = {f"C{p['C']}": [round(p["roofline"]["achieved"]), r(p["roofline"]["frac"], 3),
                                               r(p["step_ms"] * 1e3, 1)] for p in dec}
        extra["decode_128k"]["what"] = "[attn GB/s, frac of 8 TB/s, step us]"
        print("bench: extra window", file=sys.stderr, flush=True)
        win = window_steps(torch, kv, I, dev)
        detail["window_4_1020_C256_128k"] = win
        extra["window_4+1020_C256_128k"] = {"step_us": r(win["step_us"], 1), "plain_step_us": r(win["plain_step_us"], 1),
                                           "tflops": round(win["tflops"]), "GBps": round(win["algorithmic_GBps"])}
        f32 = fp32_last_step(torch, kv, I, dev)
        detail["fp32_mode_sweep_64k_last_step"] = f32
        extra["fp32_C2048_L64k"] = {"tflops": r(f32["tflops"]), "frac_fp32_peak": r(f32["frac_of_fp32_mfma_peak"], 3)}
        # the 16K fold with unrotated inputs (rotary embedding applied inside the step) and with the carried cache
        # round-tripped through int8 at every step (storage perturbation, Sec. 8)
        d = single_layer_fold("llama_16k", torch, kv, I, dev, tuning, reps=5, curve=False, rope=True)
        detail["fold_llama_16k_rope_in_step"] = d
        d2 = single_layer_fold("llama_16k", torch, kv, I, dev, tuning, reps=5, curve=False, storage_bits=8)
        detail["fold_llama_16k_int8_roundtrip"] = d2
        extra["llama_16k"]["rope_in_step_tflops"] = round(d["tflops"])
        extra["llama_16k"]["int8_roundtrip_tflops"] = round(d2["tflops"])
        result["extra"] = extra
    if args.detail:
        with open(args.detail, "w") as f:
            json.dump({"result": result, "roofline": detail_roofline, "detail": detail}, f, indent=1)
    print(json.dumps(result, separators=(",", ":")))


if __name__ == "__main__":
    main()
