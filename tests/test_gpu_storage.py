"""Storage round trip of the carried cache (Sec. 8, Discussion: bf16 -> intN -> bf16 per step): the rows a step
appends are quantised in place before its queries attend to them.  The cache must hold, bit for bit, what the
oracle's quantiser makes of the same rows; outputs are compared with the oracle's step on that cache."""
import numpy as np
import pytest
import torch

import paper_2605_12471_amd as kv
from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import fold_harness
    return fold_harness


@pytest.mark.parametrize("n_bits", [8, 4])
@pytest.mark.parametrize("Hq,Hkv,d,chunks", [(8, 2, 128, [160, 33, 1, 96]), (4, 1, 64, [100, 64, 7])])
def test_roundtrip_cache_bits_and_outputs(H, oracle, n_bits, Hq, Hkv, d, chunks):
    cfg = I.FoldConfig("store", 19, 1, Hq, Hkv, d, max(chunks), 0, "bf16")
    gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=max(chunks))
    oc = H.make_oracle(oracle, cfg, capacity=sum(chunks))
    gpu.cache.set_storage_roundtrip(n_bits)
    pos, rel = 0, []
    try:
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            if step == 1:
                k[3] = 0                                             # an all-zero row stays zero
            out = gpu.step(0, q, k, v)
            kq = oracle.storage_roundtrip(H.bits(k), n_bits)
            vq = oracle.storage_roundtrip(H.bits(v), n_bits)
            ref, _ = oc.step(H.wide(q), kq, vq, oc.len)
            err = np.abs(H.wide(out) - ref).max()
            assert err <= H.TOL["bf16"], f"step {step}: max|out-oracle| = {err}"
            x, y = H.wide(k), oracle.bf16_bits_to_f32(kq).astype(np.float64)
            rel.append(np.sqrt(((x - y) ** 2).sum() / (x ** 2).sum()))
            pos += C
        H.assert_cache_bit_exact(gpu, oc)
        print(f"int{n_bits} round trip: relative rms error of the stored K rows {np.mean(rel):.4f}")
    finally:
        gpu.close()


@pytest.mark.parametrize("n_bits", [8, 4])
def test_roundtrip_at_the_size_of_the_llama_layer(H, oracle, n_bits):
    """Benchmark config 2 (Hq=32, Hkv=8, d=128, C=2048 to 16K tokens) with the carried cache round-tripped through
    int8 / int4 at every step: sampled rows of three steps against the oracle's step on the oracle-quantised rows,
    all 16K cache rows bit-exact."""
    cfg = I.CONFIGS["llama_16k"]
    gpu = H.GpuFold(cfg)
    oc = H.make_oracle(oracle, cfg)
    gpu.cache.set_storage_roundtrip(n_bits)
    worst = 0.0
    try:
        for step in range(cfg.n_steps):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            out = gpu.step(0, q, k, v)
            kq = oracle.storage_roundtrip(H.bits(k), n_bits)
            vq = oracle.storage_roundtrip(H.bits(v), n_bits)
            rows = I.sample_rows(cfg, step, n_random=20) if step in (0, 3, cfg.n_steps - 1) else [0]
            ref, _ = oc.step(H.wide(q), kq, vq, oc.len, rows=rows)
            if len(rows) > 1:
                torch.cuda.synchronize()
                err = np.abs(H.wide(out)[rows] - ref).max()
                worst = max(worst, err)
                assert err <= H.TOL["bf16"], f"step {step}: max|out-oracle| = {err}"
        H.assert_cache_bit_exact(gpu, oc)
        print(f"\nint{n_bits} round trip at config-2 size: worst max-abs error {worst:.2e}")
    finally:
        gpu.close()


def test_roundtrip_switch_and_errors(H):
    cfg = I.FoldConfig("store_sw", 20, 1, 8, 2, 128, 64, 0, "bf16")
    g = H.GpuFold(cfg, capacity=192)
    f32 = H.GpuFold(cfg.with_(dtype="f32"), capacity=64)
    try:
        h = g.cache.handle
        assert kv.kvfold_cache_set_storage_roundtrip(h, 5) == -1
        assert kv.kvfold_cache_set_storage_roundtrip(None, 8) == -1
        assert kv.kvfold_cache_set_storage_roundtrip(f32.cache.handle, 8) == -5
        assert kv.kvfold_cache_set_storage_roundtrip(f32.cache.handle, 0) == 0
        q, k, v = I.chunk_qkv(cfg, 0, 0)
        g.step(0, q, k, v)                                            # off: bit copy
        g.cache.set_storage_roundtrip(4)
        g.step(0, q, k, v)                                            # on: quantised
        g.cache.set_storage_roundtrip(0)
        g.step(0, q, k, v)                                            # off again
        torch.cuda.synchronize()
        kd, _ = g.cache.view(0)
        kd = kd.cpu()
        want = k.transpose(0, 1)
        assert torch.equal(kd[:, 0:64], want) and torch.equal(kd[:, 128:192], want)
        assert not torch.equal(kd[:, 64:128], want)
    finally:
        g.close()
        f32.close()
