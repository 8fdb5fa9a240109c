"""The step that rotates q and k_new itself (rotary embedding at the new tokens' absolute positions, Sec. 2)
against the oracle's rotation + fold step, and against the plain step fed with inputs rotated beforehand."""
import numpy as np
import pytest
import torch

from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import fold_harness
    return fold_harness


def _rotated(oracle, x, cos, sin, dtype):
    """Oracle rotation of a torch tensor [n][heads][d]; returns (stored bits as numpy, torch tensor of the mode dtype)."""
    r = oracle.rope(x.float().numpy(), cos.numpy(), sin.numpy())
    if dtype == "bf16":
        b = oracle.f32_to_bf16_bits(r)
        return b, torch.from_numpy(b.view(np.int16)).view(torch.bfloat16)
    return r, torch.from_numpy(r)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("Hq,Hkv,d,chunks,splits,upw", [
    (8, 2, 128, [160, 160, 50, 96], 0, 0),
    (8, 2, 128, [64] * 6, 3, 2),
    (28, 4, 128, [100, 1, 33], 0, 1),
    (4, 1, 64, [128, 7, 64], 0, 0),
])
def test_rope_step_vs_oracle_and_vs_prerotated_inputs(H, oracle, dtype, Hq, Hkv, d, chunks, splits, upw):
    cfg = I.FoldConfig("rope", 16, 1, Hq, Hkv, d, max(chunks), 0, dtype)
    cap = sum(chunks)
    fused = H.GpuFold(cfg, capacity=cap, chunk_tokens=max(chunks))
    plain = H.GpuFold(cfg, capacity=cap, chunk_tokens=max(chunks))
    oc = H.make_oracle(oracle, cfg, capacity=cap)
    for g in (fused, plain):
        if splits:
            g.cache.set_tuning(0, splits)
        if upw and dtype == "bf16":
            g.cache.set_tuning(1, upw)
    pos = 0
    try:
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            cos, sin = I.rope_tables(d, pos, C)
            out_f, lse_f = fused.step(0, q, k, v, want_lse=True, rope=(cos, sin))
            # oracle: rotate, store in the mode dtype, then the ordinary fold step
            q_bits, q_rot = _rotated(oracle, q, cos, sin, dtype)
            k_bits, k_rot = _rotated(oracle, k, cos, sin, dtype)
            ref, ref_lse = oc.step(H.wide(q_rot), k_bits, H.bits(v), oc.len)
            err = np.abs(H.wide(out_f) - ref).max()
            assert err <= H.TOL[dtype], f"step {step} C={C}: max|out-oracle| = {err}"
            assert np.abs(lse_f.cpu().double().numpy().T - ref_lse).max() <= (1e-5 if dtype == "f32" else 2e-2)
            # the plain entry point on inputs rotated beforehand: the same bits
            out_p, lse_p = plain.step(0, q_rot, k_rot, v, want_lse=True)
            torch.cuda.synchronize()
            assert torch.equal(out_f.cpu(), out_p.cpu()), f"step {step}: fused and pre-rotated outputs differ"
            assert torch.equal(lse_f.cpu(), lse_p.cpu())
            pos += C
        H.assert_cache_bit_exact(fused, oc)     # the cache holds the rotated keys, bit for bit the oracle's
        H.assert_cache_bit_exact(plain, oc)
    finally:
        fused.close()
        plain.close()


def test_rope_positions_continue_across_chunks(H, oracle):
    """Rotating chunk t at positions tC + i (not at i) is what makes the fold equal to one long rotated
    sequence: outputs of a 4-chunk fold equal those of a single 256-token step with positions 0..255."""
    cfg = I.FoldConfig("rope_cont", 17, 1, 8, 2, 128, 256, 0, "f32")
    q, k, v = I.chunk_qkv(cfg, 0, 0, n_tokens=256, token_base=0)
    cos, sin = I.rope_tables(128, 0, 256)
    one = H.GpuFold(cfg, capacity=256, chunk_tokens=256)
    four = H.GpuFold(cfg, capacity=256, chunk_tokens=64)
    try:
        whole = one.step(0, q, k, v, rope=(cos, sin)).cpu()
        parts = [four.step(0, q[s:s + 64], k[s:s + 64], v[s:s + 64], rope=(cos[s:s + 64], sin[s:s + 64])).cpu()
                 for s in range(0, 256, 64)]
        assert (torch.cat(parts) - whole).abs().max() <= 2e-6
        k1, _ = one.cache.view(0)
        k4, _ = four.cache.view(0)
        assert torch.equal(k1.cpu(), k4.cpu())
    finally:
        one.close()
        four.close()


def test_rope_argument_errors(H):
    import paper_2605_12471_amd as kv
    cfg = I.FoldConfig("rope_err", 18, 1, 8, 2, 128, 64, 0, "bf16")
    g = H.GpuFold(cfg, capacity=128)
    try:
        q, k, v = (t.to("cuda:0") for t in I.chunk_qkv(cfg, 0, 0))
        out = torch.empty_like(q)
        cos, sin = (t.to("cuda:0") for t in I.rope_tables(128, 0, 64))
        h = g.cache.handle
        args = (q.data_ptr(), k.data_ptr(), v.data_ptr())
        assert kv.kvfold_step_rope(h, 0, *args, 64, 0, None, sin.data_ptr(), out.data_ptr(), None, 0) == -1
        assert kv.kvfold_step_rope(h, 0, *args, 64, 0, cos.data_ptr(), None, out.data_ptr(), None, 0) == -1
        assert kv.kvfold_step_rope(h, 0, *args, 64, 0, cos.data_ptr() + 4, sin.data_ptr(), out.data_ptr(), None, 0) == -1
        assert kv.kvfold_step_rope(h, 0, *args, 64, 5, cos.data_ptr(), sin.data_ptr(), out.data_ptr(), None, 0) == -3
        assert kv.kvfold_cache_length(h, 0) == 0
        assert kv.kvfold_step_rope(h, 0, *args, 64, 0, cos.data_ptr(), sin.data_ptr(), out.data_ptr(), None, 0) == 0
        assert kv.kvfold_cache_length(h, 0) == 64
    finally:
        g.close()


def test_rope_step_at_the_size_of_the_llama_layer(H, oracle):
    """Benchmark config 2 (Hq=32, Hkv=8, d=128, C=2048 to 16K tokens) through kvfold_step_rope, in the launch
    configuration bench.py times for its rope-in-step figure: sampled rows of three steps against the oracle
    (rotation at the absolute positions, then the ordinary fold step), cache bit-exact over all 16K rows."""
    cfg = I.CONFIGS["llama_16k"]
    gpu = H.GpuFold(cfg)
    oc = H.make_oracle(oracle, cfg)
    worst = 0.0
    try:
        for step in range(cfg.n_steps):
            pos = step * cfg.chunk
            q, k, v = I.chunk_qkv(cfg, 0, step)
            cos, sin = I.rope_tables(cfg.head_dim, pos, cfg.chunk)
            out, lse = gpu.step(0, q, k, v, want_lse=True, rope=(cos, sin))
            q_bits, q_rot = _rotated(oracle, q, cos, sin, "bf16")
            k_bits, _ = _rotated(oracle, k, cos, sin, "bf16")
            rows = I.sample_rows(cfg, step, n_random=20) if step in (0, 3, cfg.n_steps - 1) else [0]
            ref, ref_lse = oc.step(H.wide(q_rot), k_bits, H.bits(v), oc.len, rows=rows)
            if len(rows) > 1:
                torch.cuda.synchronize()
                err = np.abs(H.wide(out)[rows] - ref).max()
                worst = max(worst, err)
                assert err <= H.TOL["bf16"], f"step {step}: max|out-oracle| = {err}"
                assert np.abs(lse.cpu().double().numpy().T[rows] - ref_lse).max() <= 2e-2
        H.assert_cache_bit_exact(gpu, oc)
        print(f"\nrope at config-2 size: worst max-abs error {worst:.2e}")
    finally:
        gpu.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_rope_step_against_an_fp64_complex_rotation(H, oracle, dtype):
    """An fp64 leg that shares nothing with the fp32 rounding points chosen for the step: every (x_j, x_{j+d/2}) pair
    is rotated as a complex number in double precision, z' = z * (cos + i sin).  The keys the step leaves in the cache
    must lie within the rounding budget of that exact rotation (half a unit in the last place of the mode dtype plus
    the fp32 arithmetic error, which is relative to the operands), and the outputs
    must match the fold of the fp64-rotated inputs (keys rounded once to the mode dtype, queries unrounded)."""
    d, Hq, Hkv = 128, 8, 2
    chunks = [160, 96, 50]
    cfg = I.FoldConfig("rope64", 17, 1, Hq, Hkv, d, max(chunks), 0, dtype)
    cap = sum(chunks)
    gpu = H.GpuFold(cfg, capacity=cap, chunk_tokens=max(chunks))
    oc = H.make_oracle(oracle, cfg, capacity=cap)
    mant = 8 if dtype == "bf16" else 24          # significand bits of the mode dtype

    def rotate64(x, cos, sin):
        z = x[..., : d // 2].astype(np.float64) + 1j * x[..., d // 2:].astype(np.float64)
        z = z * (cos.astype(np.float64) + 1j * sin.astype(np.float64))[:, None, :]
        return np.concatenate([z.real, z.imag], axis=-1)

    pos = 0
    try:
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            cos, sin = I.rope_tables(d, pos, C)
            out = gpu.step(0, q, k, v, rope=(cos, sin))
            k64 = rotate64(H.wide(k), cos.numpy(), sin.numpy())                 # [C][Hkv][d], exact up to fp64 rounding
            q64 = rotate64(H.wide(q), cos.numpy(), sin.numpy())
            Kc, _ = gpu.cache.view(0)
            torch.cuda.synchronize()
            got = H.wide(Kc[:, pos:pos + C].transpose(0, 1))                    # [C][Hkv][d]
            # Error budget of the stored key against the exact rotation: the final rounding to the mode dtype (half a
            # unit in the last place) plus the step's fp32 arithmetic before it -- the sine product and the fused
            # multiply-add each round once, relative to the operands (not to the result, which may cancel):
            # at most 2^-22 (|x_j| + |x_{j+d/2}|).
            kw = H.wide(k)
            mag = np.abs(kw[..., : d // 2]) + np.abs(kw[..., d // 2:])
            mag = np.concatenate([mag, mag], axis=-1)
            big = np.maximum(np.maximum(np.abs(k64), np.abs(got)), 1e-30)
            ulp = np.exp2(np.floor(np.log2(big)) - (mant - 1))
            assert np.all(np.abs(got - k64) <= 0.5 * ulp + 2.0 ** -22 * mag), \
                f"step {step}: stored key off the fp64 rotation by more than its rounding budget"
            # outputs: the oracle's fold on the fp64-rotated inputs, keys rounded once (RNE) to the mode dtype
            if dtype == "bf16":
                k_store = oracle.f32_to_bf16_bits(k64.astype(np.float32))
            else:
                k_store = k64.astype(np.float32)
            ref, _ = oc.step(q64, k_store, H.bits(v), oc.len)
            err = np.abs(H.wide(out) - ref).max()
            assert err <= H.TOL[dtype], f"step {step}: max|out - fp64-rotated fold| = {err}"
            pos += C
    finally:
        gpu.close()
