"""GPU parity of the sink + sliding-window step (kvfold_step_window; the mask of the streaming baseline the
paper compares with, Sec. 6: a few sink tokens + a window of recent tokens, positions preserved) against the
oracle's window leg, element by element: small shapes with ragged chunks, forced splits, both wavefront shapes
and both precisions; windows that cover everything (== the plain step); the paper's 4 + 1020 configuration at
C = 256 against a 128K cache; plain and windowed steps mixed on one cache."""
import numpy as np
import pytest
import torch

from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import fold_harness
    return fold_harness


def _run_window_case(H, oracle, cfg, chunks, n_sink, window, splits=0, upw=0, profile=None, tol=None, check_lse=True):
    gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=max(chunks))
    oc = H.make_oracle(oracle, cfg, capacity=sum(chunks))
    if splits:
        gpu.cache.set_tuning(0, splits)
    if upw:
        gpu.cache.set_tuning(1, upw)
    pos, worst = 0, 0.0
    try:
        for step, C in enumerate(chunks):
            if profile:
                q, k, v = I.steered_qkv(cfg, 0, step, profile, n_tokens=C, token_base=pos)
            else:
                q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            out, lse = gpu.step(0, q, k, v, want_lse=True, window=(n_sink, window))
            ref, ref_lse = H.oracle_step(oc, q, k, v, window=(n_sink, window))
            torch.cuda.synchronize()
            err = np.abs(H.wide(out) - ref).max()
            worst = max(worst, err)
            assert err <= (tol or H.TOL[cfg.dtype]), f"step {step} C={C} pos={pos} sink={n_sink} window={window}: max|out-oracle|={err}"
            if check_lse:
                lerr = np.abs(lse.cpu().double().numpy().T - ref_lse).max()
                assert lerr <= (1e-5 if cfg.dtype == "f32" else 2e-2), f"step {step}: lse err {lerr}"
            pos += C
        H.assert_cache_bit_exact(gpu, oc)
    finally:
        gpu.close()
    return worst


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_sink,window", [(4, 100), (0, 64), (4, 1), (1, 33), (70, 50), (0, 300), (4, 1020), (130, 129)])
def test_window_small_shapes(H, oracle, dtype, n_sink, window):
    """Chunks of 96 rows with a ragged tail, up to 11 tiles of cache: windows shorter than a tile, than a unit,
    longer than the cache; sinks inside one tile, across two, none."""
    cfg = I.FoldConfig("window_small", 50, 1, 8, 2, 128, 96, 0, dtype)
    _run_window_case(H, oracle, cfg, [96, 96, 50, 96, 96, 33, 96, 96], n_sink, window)


@pytest.mark.parametrize("Hq,Hkv,d,upw", [(4, 1, 64, 1), (7, 1, 128, 2), (7, 1, 128, 1), (6, 3, 64, 2), (32, 8, 128, 2), (2, 2, 128, 2)])
def test_window_head_shapes_and_wave_shapes(H, oracle, Hq, Hkv, d, upw):
    """Group sizes 1 ... 7 (units of one workgroup spread over one to eight row blocks, so the workgroup's first
    window tile and the left-masked tiles of its wavefronts differ), both kernels."""
    cfg = I.FoldConfig("window_heads", 51, 1, Hq, Hkv, d, 256, 0, "bf16")
    _run_window_case(H, oracle, cfg, [256, 256, 256, 200, 256], 4, 200, upw=upw)
    _run_window_case(H, oracle, cfg, [256, 256, 256, 200, 256], 3, 40, upw=upw)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("splits", [2, 3, 5])
def test_window_with_split_key_range(H, oracle, dtype, splits):
    cfg = I.FoldConfig("window_split", 52, 1, 8, 2, 128, 64, 0, dtype)
    _run_window_case(H, oracle, cfg, [64] * 12 + [17], 4, 400, splits=splits)
    _run_window_case(H, oracle, cfg, [64] * 12 + [17], 66, 130, splits=splits)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_window_that_covers_the_cache_equals_the_plain_step(H, oracle, dtype):
    """window >= cache length hides nothing: outputs equal the plain step's bit for bit (same tiles, same order)."""
    cfg = I.FoldConfig("window_all", 53, 1, 8, 2, 128, 128, 0, dtype)
    chunks = [128, 128, 77, 128]
    plain = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=128)
    wind = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=128)
    try:
        pos = 0
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            a, la = plain.step(0, q, k, v, want_lse=True)
            b, lb = wind.step(0, q, k, v, want_lse=True, window=(0, 1 << 20))
            assert torch.equal(a, b) and torch.equal(la, lb), f"step {step}"
            pos += C
    finally:
        plain.close()
        wind.close()


def test_plain_and_window_steps_share_one_cache(H, oracle):
    """The windowed step appends exactly like the plain one, so the two can alternate on one cache (the cache stays
    complete: nothing is evicted)."""
    cfg = I.FoldConfig("window_mixed", 54, 1, 8, 2, 128, 128, 0, "bf16")
    gpu = H.GpuFold(cfg, capacity=6 * 128, chunk_tokens=128)
    oc = H.make_oracle(oracle, cfg, capacity=6 * 128)
    try:
        for step in range(6):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            win = (4, 150) if step % 2 else None
            out = gpu.step(0, q, k, v, window=win)
            ref, _ = H.oracle_step(oc, q, k, v, window=win)
            assert np.abs(H.wide(out) - ref).max() <= H.TOL["bf16"], f"step {step}"
        H.assert_cache_bit_exact(gpu, oc)
    finally:
        gpu.close()


def test_window_4_sinks_1020_recent_at_128k(H, oracle):
    """The paper's streaming configuration (Sec. 6: 4 sink tokens + 1020 recent tokens, C = 256, T = 128K): steps
    of 256 rows under the mask at cache lengths up to 128K, the planner's own launch geometry, every row and head
    against the oracle; the cache rows are the seeded token stream written in place."""
    L, C = 131072, 256
    cfg = I.CONFIGS["deep_chain_128k"].with_(name="window_128k", config_id=7, needle=False)
    gpu = H.GpuFold(cfg, capacity=L, chunk_tokens=C)
    oc = H.make_oracle(oracle, cfg, capacity=L)
    try:
        kd, vd = gpu.cache.view(0)
        pos = 0
        for Lp in (L // 2 - C, L - 2 * C, L - C):            # a step in the middle, then the last two of the chain
            while pos < Lp:                                    # prefix rows up to Lp, written in place
                n = min(16384, Lp - pos)
                _, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=n, token_base=pos)
                oc.append(H.bits(k), H.bits(v))
                kd[:, pos:pos + n].copy_(k.to(kd.device).transpose(0, 1))
                vd[:, pos:pos + n].copy_(v.to(vd.device).transpose(0, 1))
                pos += n
            gpu.cache.set_length(0, Lp)
            q, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=C, token_base=Lp)
            out, lse = gpu.step(0, q, k, v, want_lse=True, window=(4, 1020))
            ref, ref_lse = H.oracle_step(oc, q, k, v, window=(4, 1020))
            pos += C
            err = float(np.abs(H.wide(out) - ref).max())
            assert err <= H.TOL["bf16"], f"L_prev={Lp}: max|out-oracle| = {err}"
            assert np.abs(lse.cpu().double().numpy().T - ref_lse).max() <= 2e-2
            print(f"window 4+1020 at L_prev={Lp}: max-abs error {err}")
        H.assert_cache_bit_exact(gpu, oc)
    finally:
        gpu.close()


def test_window_argument_errors(H):
    import paper_2605_12471_amd as kv
    cfg = I.FoldConfig("window_err", 55, 1, 8, 2, 128, 64, 0, "bf16")
    gpu = H.GpuFold(cfg, capacity=128, chunk_tokens=64)
    try:
        q, k, v = (t.cuda() for t in I.chunk_qkv(cfg, 0, 0))
        out = torch.empty_like(q)
        h = gpu.cache.handle
        args = (q.data_ptr(), k.data_ptr(), v.data_ptr())
        assert kv.kvfold_step_window(h, 0, *args, 64, 0, -1, 10, out.data_ptr(), None, 0) == -1
        assert kv.kvfold_step_window(h, 0, *args, 64, 0, 4, 0, out.data_ptr(), None, 0) == -1
        assert kv.kvfold_step_window(h, 0, *args, 64, 0, 4, (1 << 30) + 1, out.data_ptr(), None, 0) == -1
        assert kv.kvfold_step_window(h, 0, *args, 64, 7, 4, 10, out.data_ptr(), None, 0) == -3
        assert gpu.cache.length(0) == 0
        assert kv.kvfold_step_window(h, 0, *args, 64, 0, 4, 10, out.data_ptr(), None, 0) == 0
        torch.cuda.synchronize()
        assert gpu.cache.length(0) == 64
    finally:
        gpu.close()


def _random_window_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 3, 4]))
        G = int(rng.choice([1, 2, 4, 7]))
        n_chunks = int(rng.integers(2, 7))
        chunks = [int(rng.choice([1, 5, 31, 32, 33, 64, 100, 128, 200, 256])) for _ in range(n_chunks)]
        dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        splits = int(rng.choice([0, 0, 2, 3]))
        upw = int(rng.choice([0, 0, 1, 2]))
        n_sink = int(rng.choice([0, 1, 4, 63, 64, 65, 130]))
        window = int(rng.choice([1, 2, 17, 32, 63, 64, 65, 100, 129, 300, 1020]))
        cases.append((dtype, Hkv * G, Hkv, d, tuple(chunks), n_sink, window, splits, upw))
    return cases


@pytest.mark.parametrize("dtype,Hq,Hkv,d,chunks,n_sink,window,splits,upw", _random_window_cases(32, 20260513))
def test_window_seeded_random_shapes(H, oracle, dtype, Hq, Hkv, d, chunks, n_sink, window, splits, upw):
    """A seeded sweep over head counts, group sizes, head dims, ragged chunk sequences (cache lengths on and off the
    tile grid), sink counts and window lengths around the tile and unit sizes, and launch shapes: every row and head of
    every windowed step against the oracle, cache bit-exact."""
    cfg = I.FoldConfig("window_rand", 56, 1, Hq, Hkv, d, max(chunks), 0, dtype)
    _run_window_case(H, oracle, cfg, list(chunks), n_sink, window, splits=splits, upw=upw if dtype == "bf16" else 0)


@pytest.mark.parametrize("profile", sorted(I.LOGIT_PROFILES))
@pytest.mark.parametrize("dtype,upw,splits", [("bf16", 2, 0), ("bf16", 1, 0), ("bf16", 2, 2), ("f32", 0, 0)])
def test_window_with_logit_jumps(H, oracle, profile, dtype, upw, splits):
    """The stress inputs of the running-max bookkeeping (logits that jump by 20 ... 100 nats, rise without end, spike,
    or start 150 nats below the rest) under a window: jumps enter and leave the window row by row, the sinks (the first
    keys, far below the rest in one profile) stay visible throughout, and a row sum that overflows sends the workgroup
    into its exact second pass with the left mask in place.  Tolerances as for the plain step's stress test."""
    cfg = I.FoldConfig("window_jumps", 57, 1, 8, 2, 128, 256, 0, dtype)
    chunks = [256, 64, 200]
    peak = max(abs(I.LOGIT_PROFILES[profile](j)) for j in range(sum(chunks)))
    _run_window_case(H, oracle, cfg, chunks, 4, 150, splits=splits, upw=upw, profile=profile, check_lse=False,
                     tol=max(1e-5, 3e-6 * peak) if dtype == "f32" else None)


def test_window_keeps_a_near_needle_and_loses_a_far_one(H, oracle):
    """The paper's comparison at the operator level (Sec. 6: the streaming baseline retrieves only while the needle is
    inside its window; the full cache retrieves at every distance).  Two needles are planted in a 10K-token fold at
    C = 256, each a key row equal to 8 * sqrt(d) * q/|q| of its own probing (row, head) of the last chunk (logit about
    90: the probe's weight sits on the needle, out = the needle's value row): one 300 tokens before its probe, one 8000
    tokens before.  The plain step retrieves both; under 4 sinks + 1020 recent tokens the near one is retrieved and
    the far one has weight exactly zero, so its probe's output is what the window alone gives."""
    import math
    cfg = I.FoldConfig("window_needles", 58, 1, 8, 2, 128, 256, 40 * 256, "bf16")
    N, C, G = cfg.n_steps, cfg.chunk, 4
    last = N - 1
    q_last, _, _ = I.chunk_qkv(cfg, 0, last)
    probes = {"near": (40, 1, 300), "far": (200, 6, 8000)}            # name: (row in the last chunk, query head, distance)
    needles = {}
    for name, (row, head, dist) in probes.items():
        pos = last * C + row - dist
        qv = q_last[row, head].float()
        needles[name] = (pos, head // G, (8.0 * math.sqrt(cfg.head_dim) * qv / qv.norm()).to(torch.bfloat16))
    plain, wind = H.GpuFold(cfg), H.GpuFold(cfg)
    oc_p, oc_w = H.make_oracle(oracle, cfg), H.make_oracle(oracle, cfg)
    rows = sorted(r for r, _, _ in probes.values())
    try:
        for step in range(N):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            k = k.clone()
            for pos, g, key in needles.values():
                if pos // C == step:
                    k[pos - step * C, g] = key
            if step < last:
                plain.step(0, q, k, v)
                wind.step(0, q, k, v)
                oc_p.append(H.bits(k), H.bits(v))
                oc_w.append(H.bits(k), H.bits(v))
            else:
                out_p = plain.step(0, q, k, v)
                out_w = wind.step(0, q, k, v, window=(4, 1020))
                ref_p, _, w_p = H.oracle_step(oc_p, q, k, v, rows=rows, want_weights=True)
                ref_w, _, w_w = H.oracle_step(oc_w, q, k, v, rows=rows, want_weights=True, window=(4, 1020))
        torch.cuda.synchronize()
        assert np.abs(H.wide(out_p)[rows] - ref_p).max() <= H.TOL["bf16"]
        assert np.abs(H.wide(out_w)[rows] - ref_w).max() <= H.TOL["bf16"]
        for name, (row, head, dist) in probes.items():
            pos, g, _ = needles[name]
            i = rows.index(row)
            v_needle = oc_p.V[g, pos]                                  # the value row stored beside the needle key
            assert int(w_p[i, head].argmax()) == pos and w_p[i, head, pos] > 0.99       # full cache: retrieved
            assert np.abs(H.wide(out_p)[row, head] - v_needle).max() <= 3e-2
            if name == "near":
                assert int(w_w[i, head].argmax()) == pos and w_w[i, head, pos] > 0.99   # inside the window: retrieved
                assert np.abs(H.wide(out_w)[row, head] - v_needle).max() <= 3e-2
            else:
                assert w_w[i, head, pos] == 0.0                                           # evicted: weight exactly zero
                assert np.abs(H.wide(out_w)[row, head] - v_needle).max() > 0.5           # ... and the output shows it
    finally:
        plain.close()
        wind.close()


@pytest.mark.parametrize("C,L_prev", [(2048, 14336), (4096, 4096), (1000, 9000)])
def test_window_long_chunks_multi_round_grids(H, oracle, C, L_prev):
    """Chunks far longer than the window (the windowed step of the 16K fold's last chunk, a 4096-row chunk, a ragged
    one off the tile grid): many workgroups per KV head, each with its own first window tile and skip, grids of up to
    two rounds; every row and head against the oracle."""
    cfg = I.CONFIGS["llama_16k"].with_(name="window_long", config_id=10, chunk=C, total_tokens=L_prev + C)
    gpu = H.GpuFold(cfg, capacity=L_prev + C, chunk_tokens=C)
    oc = H.make_oracle(oracle, cfg, capacity=L_prev + C)
    try:
        kd, vd = gpu.cache.view(0)
        _, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=L_prev, token_base=0)
        oc.append(H.bits(k), H.bits(v))
        kd[:, :L_prev].copy_(k.to(kd.device).transpose(0, 1))
        vd[:, :L_prev].copy_(v.to(vd.device).transpose(0, 1))
        gpu.cache.set_length(0, L_prev)
        q, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=C, token_base=L_prev)
        out, lse = gpu.step(0, q, k, v, want_lse=True, window=(4, 1020))
        ref, ref_lse = H.oracle_step(oc, q, k, v, window=(4, 1020))
        err = float(np.abs(H.wide(out) - ref).max())
        assert err <= H.TOL["bf16"], f"max|out-oracle| = {err}"
        assert np.abs(lse.cpu().double().numpy().T - ref_lse).max() <= 2e-2
        H.assert_cache_bit_exact(gpu, oc)
    finally:
        gpu.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_window_of_one_key_returns_the_rows_own_value(H, oracle, dtype):
    """window = 1 without sinks leaves each row its own key only, so the output is the row's own value row of its KV
    head and lse is the row's own logit.  The bf16 kernel subtracts the running maximum from the logit (weight exactly 1:
    bit-equal output); the fp32 kernel folds the scale into one fused multiply-add, whose weight is 1 to within an ulp
    and cancels against the row sum to within two roundings."""
    cfg = I.FoldConfig("window_self", 57, 1, 6, 3, 128, 512, 0, dtype)
    chunks = [512, 63, 200]
    gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=512)
    pos = 0
    try:
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            out, lse = gpu.step(0, q, k, v, want_lse=True, window=(0, 1))
            torch.cuda.synchronize()
            want = v.repeat_interleave(cfg.n_q_heads // cfg.n_kv_heads, dim=1)
            if dtype == "bf16":
                assert np.array_equal(H.bits(out), H.bits(want)), f"step {step}"
            else:
                assert (np.abs(H.wide(out) - H.wide(want)) <= 2.0 ** -22 * np.abs(H.wide(want))).all(), f"step {step}"
            logit = (H.wide(q) * H.wide(k.repeat_interleave(2, dim=1))).sum(-1) / np.sqrt(cfg.head_dim)
            assert np.abs(lse.cpu().double().numpy().T - logit).max() <= (1e-5 if dtype == "f32" else 2e-2)
            pos += C
    finally:
        gpu.close()


@pytest.mark.parametrize("n_sink,window", [(1, 1), (0, 2), (2, 1)])
def test_window_of_two_or_three_keys_holds_the_rounding_bound(H, oracle, n_sink, window):
    """With two or three visible keys the bf16 output has the size of single value entries (up to 5 for N(0,1) draws), and
    the two bf16 roundings of the path -- the weights before P.V and the output -- are each worth up to 2^-8 of that
    size.  The absolute bar of the benchmark's workloads (many keys, outputs below 1) does not apply; each element is
    held to 2^-8 (|oracle| + largest visible |value|) plus the fp32 terms."""
    cfg = I.FoldConfig("window_few", 900 + 3669, 1, 6, 3, 128, 512, 0, "bf16")
    chunks = [512, 63, 200, 32, 32, 512]
    gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=512)
    oc = H.make_oracle(oracle, cfg, capacity=sum(chunks))
    pos, vmax, worst = 0, 0.0, 0.0
    try:
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            vmax = max(vmax, float(v.float().abs().max()))
            out = gpu.step(0, q, k, v, window=(n_sink, window))
            ref, _ = H.oracle_step(oc, q, k, v, window=(n_sink, window))
            torch.cuda.synchronize()
            err = np.abs(H.wide(out) - ref)
            bound = 2.0 ** -8 * (np.abs(ref) + vmax) + 1e-3
            assert (err <= bound).all(), f"step {step}: worst excess {(err - bound).max()}"
            worst = max(worst, float(err.max()))
            pos += C
        H.assert_cache_bit_exact(gpu, oc)
        print(f"few-key window ({n_sink}, {window}): worst |out - oracle| = {worst:.4f}, largest |v| = {vmax:.2f}")
    finally:
        gpu.close()
