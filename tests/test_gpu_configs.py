"""The five benchmark configurations at full size, in the launch configuration bench.py times, against the
fp64 oracle on seeded samples of (step, row) with all heads, plus exhaustive bit-exact cache checks.

Inputs are drawn on the GPU by torch's seeded generator (paper_2605_12471_amd.inputs) and copied to the host
for the oracle; no oracle input ever comes from the HIP path."""
import math

import numpy as np
import pytest
import torch

import paper_2605_12471_amd as kv
from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def H():
    import fold_harness
    return fold_harness


def _run_sampled(H, oracle, cfg, layers_checked, n_layers=None, want_lse=False, rows_random=16, steps=None):
    """Fold cfg on the GPU (all layers, all steps); oracle on sampled steps/rows of `layers_checked`."""
    gpu = H.GpuFold(cfg, n_layers=n_layers or cfg.n_layers)
    steps = steps if steps is not None else I.sample_steps(cfg)
    ocs = {l: H.make_oracle(oracle, cfg) for l in layers_checked}
    worst, lse_out = 0.0, {}
    try:
        for step in range(cfg.n_steps):
            for layer in range(n_layers or cfg.n_layers):
                q, k, v = I.chunk_qkv(cfg, layer, step, device=DEV)
                res = gpu.step(layer, q, k, v, want_lse=want_lse)
                out, lse = res if want_lse else (res, None)
                if layer in ocs:
                    oc = ocs[layer]
                    kc, vc = k.cpu(), v.cpu()
                    if step in steps:
                        rows = I.sample_rows(cfg, step, n_random=rows_random)
                        ref, ref_lse = H.oracle_step(oc, q.cpu(), kc, vc, rows=rows)
                        err = float(np.abs(H.wide(out[rows]) - ref).max())
                        worst = max(worst, err)
                        assert err <= H.TOL[cfg.dtype], f"layer {layer} step {step}: max|out-oracle| = {err}"
                        if want_lse:
                            lerr = np.abs(lse[:, rows].cpu().double().numpy().T - ref_lse).max()
                            assert lerr <= 2e-2
                            lse_out[step] = (lse.cpu(), out.cpu())
                    else:
                        oc.append(H.bits(kc), H.bits(vc))
        for layer, oc in ocs.items():
            H.assert_cache_bit_exact(gpu, oc, layer)
    finally:
        gpu.close()
    return worst, ocs, lse_out


def test_config2_llama_layer_16k(H, oracle):
    """Hq=32, Hkv=8, d=128, bf16, C=2048, 8 steps to 16K tokens: every step, sampled rows, all heads."""
    cfg = I.CONFIGS["llama_16k"]
    worst, _, _ = _run_sampled(H, oracle, cfg, [0], steps=list(range(cfg.n_steps)), rows_random=24)
    print("config 2 worst max-abs error", worst)


def test_head_dim_64_at_benchmark_sizes(H, oracle):
    """The d = 64 instantiations of the kernels at the sizes of configs 2 and 3 (the benchmark's own shapes all have
    d = 128): C = 2048 to 16K, every step, sampled rows; C = 256 at cache lengths up to 64K in the split geometry,
    sampled steps and rows; all heads."""
    cfg = I.CONFIGS["llama_16k"].with_(name="llama_16k_d64", config_id=8, head_dim=64)
    worst, _, _ = _run_sampled(H, oracle, cfg, [0], steps=list(range(cfg.n_steps)), rows_random=16)
    cfg3 = I.CONFIGS["deep_chain_128k"].with_(name="deep_chain_64k_d64", config_id=9, head_dim=64, total_tokens=65536,
                                              needle=False)
    worst3, _, _ = _run_sampled(H, oracle, cfg3, [0], want_lse=True)
    print("d = 64: worst max-abs errors", worst, worst3)


def test_config3_deep_chain_needle_128k(H, oracle):
    """C=256, 512 chunks = 128K tokens, chain depth 511 (the paper's deepest operating point, Sec. 5),
    with a planted needle: a key row in chunk 0 equal to 8 * q/||q|| for a query row of the last chunk."""
    cfg = I.CONFIGS["deep_chain_128k"]
    spec = I.needle_spec(cfg)
    last = cfg.n_steps - 1
    worst, ocs, lse_out = _run_sampled(H, oracle, cfg, [0], want_lse=True)
    oc = ocs[0]
    # --- retrieval weight of the needle row, oracle side
    q_last, _, _ = I.chunk_qkv(cfg, 0, last, device=DEV)
    row = spec.query_row - last * cfg.chunk
    _, _, w = oc.attend(H.wide(q_last), last * cfg.chunk, rows=[row], want_weights=True)
    w = w[0, spec.query_head]
    assert int(w.argmax()) == spec.key_pos                               # retrieval lands on the planted row
    runner_up = np.partition(w, -2)[-2]
    assert w[spec.key_pos] > 20 * runner_up
    # closed form: one logit ~8 among n-1 logits ~ N(0,1): weight ~ e^8 / (e^8 + n e^{1/2})
    n = spec.query_row + 1
    expect = math.exp(8) / (math.exp(8) + n * math.exp(0.5))
    assert 0.5 * expect < w[spec.key_pos] < 2.0 * expect
    # --- GPU side: weight recovered from the kernel's log-sum-exp and one dot product
    lse, _ = lse_out[last]
    kd = oc.K[spec.query_head // 4, spec.key_pos]
    logit = float(H.wide(q_last)[row, spec.query_head] @ kd) / math.sqrt(cfg.head_dim)
    w_gpu = math.exp(logit - float(lse[spec.query_head, row]))
    assert abs(w_gpu - w[spec.key_pos]) <= 2e-2 * w[spec.key_pos]
    print("config 3 worst max-abs error", worst, "needle weight", w[spec.key_pos], "gpu", w_gpu, "closed form", expect)


def test_config4_full_stack_32_layers_128k(H, oracle):
    """32 independent layers, C=4096, 32 steps each, 16 GiB of K/V resident; three layers checked, the others
    run alongside (cross-layer isolation: a layer's output and cache must not depend on its neighbours')."""
    cfg = I.CONFIGS["full_stack_128k"]
    free, _ = torch.cuda.mem_get_info()
    assert free > 24 * 2 ** 30, "needs the 16 GiB cache plus staging"
    # sample of the measurement plan: steps {0, 1, 2, 16, 30, 31} + 8 seeded ones, rows {0, 1, C/2, C-2, C-1} + 16
    # seeded ones per step, all 32 heads, on layers 0, 13 and 31
    worst, _, _ = _run_sampled(H, oracle, cfg, [0, 13, 31])
    print("config 4 worst max-abs error", worst)


def test_config5_chunk_size_and_precision_sweep(H, oracle):
    """Hq=28, Hkv=4 (G=7), 64K tokens, C in {128, 512, 2048, 8192} x {fp32, bf16} on one token stream:
    every run against the oracle at sampled positions; drift between chunk sizes and between precisions."""
    base = I.CONFIGS["sweep_64k"]
    T = base.total_tokens
    g = torch.Generator().manual_seed(5)
    pos = sorted(set([0, 1, 127, 128, 8191, 8192, T // 2, T - 2, T - 1] + torch.randint(0, T, (40,), generator=g).tolist()))
    outs = {}
    for dtype in ("f32", "bf16"):
        for C in (128, 512, 2048, 8192):
            cfg = base.with_(chunk=C, dtype=dtype)
            gpu = H.GpuFold(cfg)
            res = torch.empty((T, cfg.n_q_heads, cfg.head_dim), dtype=I.torch_dtype(dtype), device=DEV)
            try:
                for step in range(cfg.n_steps):
                    q, k, v = I.chunk_qkv(cfg, 0, step, device=DEV)
                    q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
                    gpu.cache.step(0, q, k, v, res[step * C:(step + 1) * C])
                torch.cuda.synchronize()
            finally:
                gpu.close()
            outs[(dtype, C)] = res
    # oracle once per precision (the inputs differ by their rounding), independent of C
    for dtype in ("f32", "bf16"):
        cfg = base.with_(chunk=8192, dtype=dtype)
        oc = H.make_oracle(oracle, cfg)
        ref = {}
        for step in range(cfg.n_steps):
            q, k, v = I.chunk_qkv(cfg, 0, step, device=DEV)
            rows = [p_ - step * 8192 for p_ in pos if step * 8192 <= p_ < (step + 1) * 8192]
            if rows:
                r, _ = H.oracle_step(oc, q.cpu(), k.cpu(), v.cpu(), rows=rows)
                for i, rr in enumerate(rows):
                    ref[step * 8192 + rr] = r[i]
            else:
                oc.append(H.bits(k.cpu()), H.bits(v.cpu()))
        refm = np.stack([ref[p_] for p_ in pos])
        for C in (128, 512, 2048, 8192):
            got = H.wide(outs[(dtype, C)][pos])
            err = np.abs(got - refm).max()
            assert err <= H.TOL[dtype], f"{dtype} C={C}: {err}"
    # drift between chunk sizes (same precision) and between precisions (same chunk size), all tokens
    report = {}
    for dtype, lim in (("f32", 1e-5), ("bf16", 2 ** -5 + 1e-6)):   # bf16: at most one ulp of |out| < 8
        ref_run = outs[(dtype, 8192)].float()
        for C in (128, 512, 2048):
            d = float((outs[(dtype, C)].float() - ref_run).abs().max())
            report[f"{dtype} C={C} vs C=8192"] = d
            assert d <= lim
    for C in (128, 512, 2048, 8192):
        d = float((outs[("f32", C)] - outs[("bf16", C)].float()).abs().max())
        report[f"fp32 vs bf16 C={C}"] = d
        assert d <= 6e-2   # input rounding of q, k, v to bf16 dominates
    print("config 5 drift report", report)


@pytest.mark.parametrize("C", [1, 4, 16])
def test_decode_shaped_steps_against_128k_cache(H, oracle, C):
    """Steps of 1..16 tokens against a 128K cache of the Llama-shaped layer (the decode that follows the
    chain, Sec. 4): 64 prefix splits + merge, every row and head against the oracle, cache bit-exact."""
    L = 131072
    cfg = I.CONFIGS["llama_16k"].with_(name="decode_128k", config_id=6, chunk=C, total_tokens=L)
    Lp = L - C
    gpu = H.GpuFold(cfg, capacity=L, chunk_tokens=C)
    oc = H.make_oracle(oracle, cfg, capacity=L)
    try:
        kd, vd = gpu.cache.view(0)                       # [Hkv][capacity][d]
        for t0 in range(0, Lp, 16384):                   # prefix rows: the seeded token stream, written in place
            n = min(16384, Lp - t0)
            _, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=n, token_base=t0)
            oc.append(H.bits(k), H.bits(v))
            kd[:, t0:t0 + n].copy_(k.to(DEV).transpose(0, 1))
            vd[:, t0:t0 + n].copy_(v.to(DEV).transpose(0, 1))
        gpu.cache.set_length(0, Lp)
        assert gpu.cache.plan(C, L)[1] > 1               # the prefix is split
        q, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=C, token_base=Lp)
        out, lse = gpu.step(0, q, k, v, want_lse=True)
        ref, ref_lse = H.oracle_step(oc, q, k, v)
        err = float(np.abs(H.wide(out) - ref).max())
        assert err <= H.TOL["bf16"], f"C={C}: max|out-oracle| = {err}"
        assert np.abs(lse.cpu().double().numpy().T - ref_lse).max() <= 2e-2
        H.assert_cache_bit_exact(gpu, oc)
        print(f"decode-shaped C={C}: max-abs error {err}")
    finally:
        gpu.close()


def test_largest_cache_of_one_head(H, oracle):
    """The largest cache one KV head may have (rows x row bytes just under 2^32: 16,777,215 tokens at d=128
    bf16, 8.6 GB for K and V), a step at its very end.  The oracle cannot walk 16.7M keys per row, so the far
    prefix is given a closed form: every far K row is the same vector (one logit s_far per query row), far V
    rows repeat a seeded block of 4099 rows (a prime, so a row offset that wrapped at 2^32 bytes = 2^24 rows
    would shift the pattern); the queries are steered so that far and near keys weigh about the same.  Then
        out = (e^s_far * sum_far V + Z_near * out_near) / (N_far e^s_far + Z_near),
    with out_near and Z_near = exp(lse_near) from the oracle on the last 1000 prefix rows plus the chunk.
    Checks the 32-bit row offsets at their limit, every far key visited exactly once, the appended rows
    bit-exact at the end of the buffer and nothing written at its start."""
    free, _ = torch.cuda.mem_get_info()
    if free < 24 * 2**30:
        pytest.skip("needs 24 GiB of free device memory")
    d, Hq, Hkv, C, W, P = 128, 2, 1, 256, 1000, 4099
    cap = (1 << 24) - 1
    cfg = I.FoldConfig("largest", 41, 1, Hq, Hkv, d, C, cap, "bf16")
    n_far = cap - C - W
    gpu = H.GpuFold(cfg, capacity=cap, chunk_tokens=C)
    try:
        qn, kn, vn = I.chunk_qkv(cfg, 0, 0, n_tokens=W, token_base=0)          # near rows
        q, k, v = I.chunk_qkv(cfg, 0, 1, n_tokens=C, token_base=W)             # the chunk
        base = I.chunk_qkv(cfg, 0, 2, n_tokens=P, token_base=100000)[2][:, 0].contiguous()   # [P][d] bf16
        # every query gets a component along a seeded unit vector u and the far key lies against it, so that
        # s_far is about -7 nats for every row and the 16.7M far keys weigh about as much as the 1256 near ones
        u = I.chunk_qkv(cfg, 0, 3, n_tokens=1, token_base=200000)[1][0, 0].float()    # (streams are keyed by token index)
        u = u / u.norm()
        q = (q.float() + 2.0 * math.sqrt(d) * u).to(torch.bfloat16)
        kf = (-3.5 * u + 0.05 * I.chunk_qkv(cfg, 0, 4, n_tokens=1, token_base=200001)[1][0, 0].float()).to(torch.bfloat16)  # [d]
        K, V = gpu.cache.view(0)                                                # [Hkv][cap][d]
        dev = K.device
        K[0, :n_far] = kf.to(dev)
        idx = torch.arange(n_far, device=dev) % P
        V[0, :n_far] = base.to(dev)[idx]
        del idx
        K[0, n_far:n_far + W] = kn[:, 0].to(dev)
        V[0, n_far:n_far + W] = vn[:, 0].to(dev)
        head_k, head_v = K[0, :4].clone(), V[0, :4].clone()
        gpu.cache.set_length(0, cap - C)
        out, lse = gpu.step(0, q, k, v, want_lse=True)
        torch.cuda.synchronize()
        assert gpu.cache.length(0) == cap
        # appended rows at the very end, bit for bit; the start of the buffer untouched
        assert np.array_equal(H.bits(K[0, cap - C:]), H.bits(k[:, 0])) and np.array_equal(H.bits(V[0, cap - C:]), H.bits(v[:, 0]))
        assert torch.equal(K[0, :4], head_k) and torch.equal(V[0, :4], head_v)
        # near part through the oracle
        oc = H.make_oracle(oracle, cfg, capacity=W + C)
        H.oracle_step(oc, qn, kn, vn)
        out_near, lse_near = H.oracle_step(oc, q, k, v)                         # [C][Hq][d], [C][Hq]
        # far part in closed form (fp64)
        s_far = (H.wide(q) @ kf.double().numpy()) / np.sqrt(d)                  # [C][Hq]
        b64 = base.double().numpy()
        sum_far_v = (n_far // P) * b64.sum(0) + b64[: n_far % P].sum(0)         # [d]
        z_near = np.exp(lse_near)
        den = n_far * np.exp(s_far) + z_near
        want = (np.exp(s_far)[..., None] * sum_far_v[None, None, :] + z_near[..., None] * out_near) / den[..., None]
        err = np.abs(H.wide(out) - want).max()
        print(f"\nlargest cache: {cap} tokens, far weight share {float((n_far * np.exp(s_far) / den).mean()):.3f}, max|out-closed form|={err:.2e}")
        assert err <= H.TOL["bf16"]
        share = n_far * np.exp(s_far) / den
        assert 0.15 < share.mean() < 0.85, "far and near keys should both matter"
        lerr = np.abs(lse.cpu().double().numpy().T - np.log(den)).max()
        assert lerr <= 2e-2
        # one row beyond the end is refused
        with pytest.raises(kv.KvFoldError):
            gpu.step(0, q[:1], k[:1], v[:1])
    finally:
        gpu.close()


def test_multi_needle_retrieval_across_chain_depths(H, oracle):
    """Several needles at once (the paper's multi-needle stress test, Sec. 5, at the operator level): eight key
    rows planted at seeded positions in eight different chunks of a 32K-token fold (C=512, chain depth 63), each
    equal to 8 * q/||q|| for its own probing (row, head) of the last chunk.  Every probe has to retrieve its own
    needle through the carried cache -- the weight argmax, its size against the closed form, the GPU's weight
    recovered from the kernel's log-sum-exp -- and the probing rows match the oracle."""
    cfg = I.FoldConfig("multi_needle", 45, 1, 32, 8, 128, 512, 32768, "bf16")
    N, C, G = cfg.n_steps, cfg.chunk, cfg.n_q_heads // cfg.n_kv_heads
    last = N - 1
    rng = np.random.default_rng(20260512)
    n_needles = 8
    chunks = [0, 7, 15, 24, 33, 42, 51, 60]                       # one needle per listed chunk
    kv_heads = rng.permutation(cfg.n_kv_heads)[:n_needles]         # distinct KV heads: the probes do not collide
    needles = []
    q_last, _, _ = I.chunk_qkv(cfg, 0, last)
    for i in range(n_needles):
        head = int(kv_heads[i]) * G + int(rng.integers(0, G))
        row = int(rng.integers(0, C))
        pos = chunks[i] * C + int(rng.integers(0, C))
        qv = q_last[row, head].float()
        key = (8.0 * qv / qv.norm()).to(torch.bfloat16)
        needles.append((pos, row, head, key))
    gpu = H.GpuFold(cfg)
    oc = H.make_oracle(oracle, cfg)
    probe_rows = sorted({r for _, r, _, _ in needles})
    try:
        for step in range(N):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            k = k.clone()
            for pos, _, head, key in needles:
                if pos // C == step:
                    k[pos - step * C, head // G] = key
            out, lse = gpu.step(0, q, k, v, want_lse=True)
            if step < last:
                H.oracle_step(oc, q, k, v, rows=[0])
        ref, ref_lse, w = H.oracle_step(oc, q, k, v, rows=probe_rows, want_weights=True)
        torch.cuda.synchronize()
        err = np.abs(H.wide(out)[probe_rows] - ref).max()
        assert err <= H.TOL["bf16"]
        H.assert_cache_bit_exact(gpu, oc)
        lse = lse.cpu().double().numpy()                          # [Hq][C]
        for pos, row, head, key in needles:
            wi = w[probe_rows.index(row), head]
            assert int(wi.argmax()) == pos, f"needle at {pos} (chunk {pos // C}) not retrieved by row {row} head {head}"
            n_keys = last * C + row + 1
            logit = float(H.wide(q_last)[row, head] @ key.double().numpy()) / math.sqrt(cfg.head_dim)   # 8 |q| / sqrt(d)
            expect = math.exp(logit) / (math.exp(logit) + n_keys * math.exp(0.5))      # among n logits ~ N(0, 1)
            assert 0.5 * expect < wi[pos] < 2.0 * expect
            w_gpu = math.exp(logit - lse[head, row])
            assert abs(w_gpu - wi[pos]) <= 2e-2 * wi[pos]
        print(f"\nmulti-needle: 8 needles over chain depth {last}, max|out-oracle| on the probing rows {err:.2e}, "
              f"weights {[round(float(w[probe_rows.index(r), h][p]), 3) for p, r, h, _ in needles]}")
    finally:
        gpu.close()
