"""GPU parity of the HIP fold step against the fp64 oracle, element by element, on sizes the oracle
finishes in seconds but that span several tiles, ragged tails, splits and both wave shapes."""
import numpy as np
import pytest
import torch

from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import fold_harness
    return fold_harness


def _run_case(H, oracle, cfg, chunks, splits=0, upw=0, check_lse=True, profile=None, tol=None, pair=0):
    gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=max(chunks))
    oc = H.make_oracle(oracle, cfg, capacity=sum(chunks))
    if splits:
        gpu.cache.set_tuning(0, splits)
    if upw:
        gpu.cache.set_tuning(1, upw)
    if pair:
        gpu.cache.set_tuning(2, pair)   # 1 = never, 2 = always pair an early and a late row block in a wavefront
    pos, worst = 0, 0.0
    try:
        for step, C in enumerate(chunks):
            if profile:
                q, k, v = I.steered_qkv(cfg, 0, step, profile, n_tokens=C, token_base=pos)
            else:
                q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            out, lse = gpu.step(0, q, k, v, want_lse=True)
            ref, ref_lse = H.oracle_step(oc, q, k, v)
            torch.cuda.synchronize()
            err = np.abs(H.wide(out) - ref).max()
            worst = max(worst, err)
            assert err <= (tol or H.TOL[cfg.dtype]), f"step {step} C={C} pos={pos}: max|out-oracle|={err}"
            if check_lse:
                lerr = np.abs(lse.cpu().double().numpy().T - ref_lse).max()
                assert lerr <= (1e-5 if cfg.dtype == "f32" else 2e-2), f"step {step}: lse err {lerr}"
            pos += C
        H.assert_cache_bit_exact(gpu, oc)
    finally:
        gpu.close()
    return worst


def test_config1_tiny_fp32_vs_oracle_and_monolithic(H, oracle):
    """Benchmark config 1: 1 layer, Hq=4, Hkv=1, d=64, C=128, 4 chunks, fp32, tolerance 1e-5."""
    cfg = I.CONFIGS["tiny_f32"]
    gpu = H.GpuFold(cfg)
    oc = H.make_oracle(oracle, cfg)
    outs, Q, K, V = [], [], [], []
    try:
        for step in range(cfg.n_steps):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            out = gpu.step(0, q, k, v)
            ref, _ = H.oracle_step(oc, q, k, v)
            assert np.abs(H.wide(out) - ref).max() <= 1e-5
            outs.append(H.wide(out)); Q.append(H.wide(q)); K.append(H.wide(k)); V.append(H.wide(v))
        H.assert_cache_bit_exact(gpu, oc)
    finally:
        gpu.close()
    mono, _ = oracle.monolithic_causal_attention(np.concatenate(Q), np.concatenate(K), np.concatenate(V))
    assert np.abs(np.concatenate(outs) - mono).max() <= 1e-5


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("Hq,Hkv,d", [(4, 1, 64), (8, 2, 128), (7, 1, 128), (6, 3, 64)])
def test_ragged_chunks(H, oracle, dtype, Hq, Hkv, d):
    cfg = I.FoldConfig("ragged", 10, 1, Hq, Hkv, d, 100, 0, dtype)
    _run_case(H, oracle, cfg, [100, 1, 33, 64, 7, 95])


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("splits", [2, 3, 5])
def test_forced_splits(H, oracle, dtype, splits):
    cfg = I.FoldConfig("splits", 11, 1, 8, 2, 128, 64, 0, dtype)
    _run_case(H, oracle, cfg, [64] * 3 + [40] + [64] * 20, splits=splits)


@pytest.mark.parametrize("upw", [1, 2])
@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (28, 4), (4, 4)])
def test_units_per_wave_bf16(H, oracle, upw, Hq, Hkv):
    cfg = I.FoldConfig("upw", 12, 1, Hq, Hkv, 128, 160, 0, "bf16")
    _run_case(H, oracle, cfg, [160, 160, 50, 160], upw=upw)


@pytest.mark.parametrize("profile", sorted(I.LOGIT_PROFILES))
@pytest.mark.parametrize("dtype,upw,splits", [("bf16", 2, 0), ("bf16", 1, 0), ("bf16", 2, 2), ("f32", 0, 0)])
def test_logit_jumps_and_overflow(H, oracle, profile, dtype, upw, splits):
    """Logits that jump by 20 ... 100 nats inside the prefix, inside the causal part, rise without end, or
    start 150 nats below the rest: the reference of the online softmax has to follow (sum-driven shift, exact
    second pass after an overflow, exact row max at the causal horizon, a first reference far below zero).  lse is not compared: the steering component of a
    logit of g nats carries a rounding error of g * 2^-9 that is common to all keys (it cancels in out).
    fp32: a dot product of d fp32 terms that sums to a logit of g nats carries a rounding error of about
    g * sqrt(d) * 2^-24 nats (7e-7 g at d=128), the weights inherit it as a relative error and the output as
    that times |v| <= 4: the 1e-5 of the N(0,1) workloads (|logit| < 10) becomes 3e-6 g for these."""
    cfg = I.FoldConfig("jumps", 15, 1, 8, 2, 128, 256, 0, dtype)
    chunks = [256, 64, 200]
    peak = max(abs(I.LOGIT_PROFILES[profile](j)) for j in range(sum(chunks)))
    _run_case(H, oracle, cfg, chunks, splits=splits, upw=upw, check_lse=False, profile=profile,
              tol=max(1e-5, 3e-6 * peak) if dtype == "f32" else None)


def test_isolated_chunk_equals_plain_causal(H, oracle):
    """Empty cache (the paper's ISOLATED condition, Sec. 2): the step is plain causal attention."""
    cfg = I.FoldConfig("iso", 13, 1, 8, 4, 128, 256, 0, "bf16")
    q, k, v = I.chunk_qkv(cfg, 0, 0)
    gpu = H.GpuFold(cfg, capacity=256)
    try:
        out = gpu.step(0, q, k, v)
        mono, _ = oracle.monolithic_causal_attention(H.wide(q), H.wide(k), H.wide(v))
        assert np.abs(H.wide(out) - mono).max() <= 2e-2
    finally:
        gpu.close()


def test_layers_are_independent(H, oracle):
    cfg = I.FoldConfig("layers", 14, 3, 8, 2, 128, 64, 0, "bf16")
    gpu = H.GpuFold(cfg, capacity=192)
    ocs = [H.make_oracle(oracle, cfg, capacity=192) for _ in range(3)]
    try:
        for step in range(3):
            for layer in (2, 0, 1):
                q, k, v = I.chunk_qkv(cfg, layer, step)
                out = gpu.step(layer, q, k, v)
                ref, _ = H.oracle_step(ocs[layer], q, k, v)
                assert np.abs(H.wide(out) - ref).max() <= 2e-2
        for layer in range(3):
            H.assert_cache_bit_exact(gpu, ocs[layer], layer)
    finally:
        gpu.close()


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        d = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 3, 4]))
        G = int(rng.choice([1, 2, 4, 7]))
        n_chunks = int(rng.integers(1, 5))
        chunks = [int(rng.choice([1, 5, 31, 32, 33, 64, 100, 128, 200, 256])) for _ in range(n_chunks)]
        dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        splits = int(rng.choice([0, 0, 2, 4]))
        upw = int(rng.choice([0, 0, 1, 2]))
        cases.append((dtype, Hkv * G, Hkv, d, tuple(chunks), splits, upw))
    return cases


@pytest.mark.parametrize("dtype,Hq,Hkv,d,chunks,splits,upw", _random_cases(28, 20260512))
def test_seeded_random_shapes(H, oracle, dtype, Hq, Hkv, d, chunks, splits, upw):
    """A seeded sweep over head counts, group sizes, head dims, ragged chunk sequences and launch shapes: every
    row and head of every step against the oracle, cache bit-exact."""
    cfg = I.FoldConfig("rand", 21, 1, Hq, Hkv, d, max(chunks), 0, dtype)
    _run_case(H, oracle, cfg, list(chunks), splits=splits, upw=upw if dtype == "bf16" else 0)


@pytest.mark.parametrize("dtype,Hq,Hkv,d", [("bf16", 48, 24, 128), ("bf16", 64, 64, 64), ("bf16", 10, 5, 128),
                                             ("bf16", 12, 6, 64), ("f32", 32, 16, 64)])
def test_more_kv_heads_than_xcds_and_odd_head_counts(H, oracle, dtype, Hq, Hkv, d):
    """KV head counts above 8 (several heads per XCD) and counts that do not divide 8 (contiguous id ranges)."""
    cfg = I.FoldConfig("heads", 27, 1, Hq, Hkv, d, 200, 0, dtype)
    _run_case(H, oracle, cfg, [128, 200, 33, 64])


@pytest.mark.parametrize("d,upw", [(64, 2), (64, 1), (128, 2)])
def test_long_prefix_small_case(H, oracle, d, upw):
    """4K tokens in chunks of 512: enough tiles for the unmasked main loop, the ring to wrap many times and the
    clamp-free refill path, on both head dims and both wave shapes."""
    cfg = I.FoldConfig("longish", 22, 1, 8, 2, d, 512, 0, "bf16")
    _run_case(H, oracle, cfg, [512] * 8, upw=upw)


@pytest.mark.parametrize("Hq,Hkv,d,chunks", [
    (8, 2, 128, [256, 256, 100, 256]),        # 4 heads x 8 blocks per KV head: full pairs
    (28, 4, 128, [160, 33, 160]),             # G = 7: 35 units per head, an odd number (the middle one pairs with itself)
    (4, 4, 128, [96, 200, 64]),               # G = 1: few units, workgroups partly empty
    (8, 2, 64, [256, 130, 256]),
    (6, 3, 128, [32, 31, 1, 64]),             # chunks of one block and less
])
@pytest.mark.parametrize("pair", [1, 2])
def test_unit_pairing(H, oracle, Hq, Hkv, d, chunks, pair):
    """Two-unit kernel with an early and a late row block per wavefront (and without): the late unit finishes
    alone once every further key lies beyond the early unit's last row."""
    cfg = I.FoldConfig("pairing", 23, 1, Hq, Hkv, d, max(chunks), 0, "bf16")
    _run_case(H, oracle, cfg, chunks, upw=2, pair=pair)


@pytest.mark.parametrize("splits", [2, 3, 5])
@pytest.mark.parametrize("Hq,Hkv,d,chunks", [
    (8, 2, 128, [256, 256, 100, 256]),
    (28, 4, 128, [160, 33, 160]),
    (4, 2, 64, [96, 300, 64]),
])
def test_unit_pairing_with_prefix_splits(H, oracle, Hq, Hkv, d, chunks, splits):
    """Pairing together with a split key range: pieces that end before the early unit's horizon run both
    units throughout, pieces that begin beyond it run the late unit alone from their first tile."""
    cfg = I.FoldConfig("pairsplit", 24, 1, Hq, Hkv, d, max(chunks), 0, "bf16")
    _run_case(H, oracle, cfg, chunks, splits=splits, upw=2, pair=2)


@pytest.mark.parametrize("profile", ["step100", "stairs", "late"])
def test_unit_pairing_with_logit_jumps(H, oracle, profile):
    cfg = I.FoldConfig("jumps", 15, 1, 8, 2, 128, 256, 0, "bf16")
    _run_case(H, oracle, cfg, [256, 64, 200], upw=2, check_lse=False, profile=profile, pair=2)
