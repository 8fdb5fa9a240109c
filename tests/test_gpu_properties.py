"""Properties of the HIP fold step that hold at any size, plus the error paths that need a live cache."""
import ctypes

import numpy as np
import pytest
import torch

import paper_2605_12471_amd as kv
from paper_2605_12471_amd import binding
from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import fold_harness
    return fold_harness


def _fold(H, cfg, chunks, mutate=None, sync_each=True, tuning=None):
    """Run a fold; returns list of per-step outputs (CPU tensors) and the GpuFold (caller closes)."""
    gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=max(chunks))
    for k_, v_ in (tuning or {}).items():
        gpu.cache.set_tuning(k_, v_)
    outs, pos = [], 0
    for step, C in enumerate(chunks):
        q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
        if mutate:
            q, k, v = mutate(step, pos, q, k, v)
        out = gpu.step(0, q, k, v)
        if sync_each:
            torch.cuda.synchronize()
        outs.append(out)
        pos += C
    torch.cuda.synchronize()
    return [o.cpu() for o in outs], gpu


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_gqa_group_isolation(H, dtype):
    """Changing the V rows of one KV head changes exactly its G query heads, nothing else (bit for bit)."""
    cfg = I.FoldConfig("gqa", 20, 1, 12, 3, 128, 96, 0, dtype)
    chunks = [96, 96, 40]
    base, g0 = _fold(H, cfg, chunks); g0.close()

    def bump(step, pos, q, k, v):
        v = v.clone(); v[:, 1] += 1.0
        return q, k, v
    pert, g1 = _fold(H, cfg, chunks, mutate=bump); g1.close()
    for b, p_ in zip(base, pert):
        same = [h for h in range(12) if torch.equal(b[:, h], p_[:, h])]
        assert same == [0, 1, 2, 3, 8, 9, 10, 11]
        # weights sum to one, so the bumped heads move by the bump (up to rounding)
        assert (p_[:, 4:8].double() - b[:, 4:8].double() - 1.0).abs().max() < (3e-2 if dtype == "bf16" else 1e-5)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_no_causal_leak(H, dtype):
    """Perturbing key/value row j leaves every output row at a position < j unchanged bit for bit."""
    cfg = I.FoldConfig("leak", 21, 1, 8, 2, 128, 128, 0, dtype)
    chunks = [128, 128, 128]
    base, g0 = _fold(H, cfg, chunks); g0.close()
    j = 128 + 77   # inside chunk 1

    def poke(step, pos, q, k, v):
        if pos <= j < pos + k.shape[0]:
            k, v = k.clone(), v.clone()
            k[j - pos] *= -3.0
            v[j - pos] += 5.0
        return q, k, v
    pert, g1 = _fold(H, cfg, chunks, mutate=poke); g1.close()
    b, p_ = torch.cat(base), torch.cat(pert)
    assert torch.equal(b[:j], p_[:j])
    assert not torch.equal(b[j:], p_[j:])
    assert (b[j:].double() - p_[j:].double()).abs().flatten(1).max(1).values.min() > 0   # every later row moved


def test_determinism_and_stream_order(H):
    """Same inputs give bit-identical outputs; steps enqueued back to back without host syncs equal synced steps."""
    cfg = I.FoldConfig("det", 22, 1, 32, 8, 128, 256, 0, "bf16")
    chunks = [256] * 6
    a, g0 = _fold(H, cfg, chunks, sync_each=True); g0.close()
    b, g1 = _fold(H, cfg, chunks, sync_each=False); g1.close()
    for x, y in zip(a, b):
        assert torch.equal(x, y)
    # on a side stream as well
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        c, g2 = _fold(H, cfg, chunks, sync_each=False)
    g2.close()
    for x, y in zip(a, c):
        assert torch.equal(x, y)


@pytest.mark.parametrize("Hq,Hkv,d,chunks,splits", [
    (32, 8, 128, [256] * 5, 0),
    (8, 2, 128, [64, 128, 64, 192, 64], 3),          # split launches: pieces that end before the chunk begins
    (28, 4, 64, [128, 128, 16, 48, 64, 33, 31, 64], 0),   # lengths that leave and regain a multiple of 64
    (4, 4, 128, [512, 64, 1, 63, 512], 2),
    (32, 8, 128, [1000, 1, 1, 16, 5, 1], 0),          # decode-shaped steps at lengths off the tile grid
    (8, 2, 128, [777, 3, 100, 1, 64], 4),             # ... with the straddling tile inside a split piece
])
def test_fused_append_equals_separate_append(H, Hq, Hkv, d, chunks, splits):
    """bf16: the attention kernel copies the chunk's rows into the cache itself and reads the chunk's own rows from
    k_new / v_new (a tile that straddles the cache's end is filled from both sides); switched off (tuning knob)
    the separate append kernel runs first.  Same bits either way, outputs and cache."""
    cfg = I.FoldConfig("fused", 26, 1, Hq, Hkv, d, max(chunks), 0, "bf16")
    res = []
    for knob in (0, 1):
        gpu = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=max(chunks))
        gpu.cache.set_tuning(kv.TUNE_FUSED_APPEND, knob)
        if splits:
            gpu.cache.set_tuning(kv.TUNE_SPLITS, splits)
        outs, pos = [], 0
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            outs.append(gpu.step(0, q, k, v).clone())
            pos += C
        torch.cuda.synchronize()
        K, V = gpu.cache.view(0)
        res.append((outs, K[:, :pos].clone(), V[:, :pos].clone()))
        gpu.close()
    for a, b in zip(res[0][0], res[1][0]):
        assert torch.equal(a, b)
    assert torch.equal(res[0][1], res[1][1]) and torch.equal(res[0][2], res[1][2])


@pytest.mark.parametrize("C,L_prev,dtype,mode", [(256, 1024, "bf16", "plain"), (16, 4000, "bf16", "plain"), (64, 512, "f32", "plain"),
                                                 (256, 3000, "bf16", "window"), (16, 4000, "bf16", "rope"), (100, 1000, "f32", "window")])
def test_step_under_graph_capture(H, C, L_prev, dtype, mode):
    """A step allocates nothing and only enqueues kernels, so it can be captured into a HIP graph: several
    replays, with eager work and synchronisations between them, give the bits of the eager step (unsplit and
    split launches: append, attention, merge; the plain step, the sink + sliding-window step and the step that
    applies the rotary embedding itself)."""
    cfg = I.FoldConfig("graph", 25, 1, 8, 2, 128, C, 0, dtype)
    gpu = H.GpuFold(cfg, capacity=L_prev + C, chunk_tokens=max(C, 256))
    try:
        pos = 0
        while pos < L_prev:                                   # build the prefix eagerly
            n = min(256, L_prev - pos)
            q, k, v = I.chunk_qkv(cfg, 0, pos // 256, n_tokens=n, token_base=pos)
            gpu.step(0, q, k, v)
            pos += n
        q, k, v = (t.to(gpu.dev).contiguous() for t in I.chunk_qkv(cfg, 0, 99, n_tokens=C, token_base=L_prev))
        out = torch.empty_like(q)
        lse = torch.empty((cfg.n_q_heads, C), dtype=torch.float32, device=gpu.dev)
        kw = {}
        if mode == "window":
            kw["window"] = (4, 300)
        elif mode == "rope":
            kw["rope"] = tuple(t.to(gpu.dev).contiguous() for t in I.rope_tables(cfg.head_dim, L_prev, C))
        gpu.cache.step(0, q, k, v, out, lse=lse, **kw)
        torch.cuda.synchronize()
        want, want_lse = out.clone(), lse.clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        gpu.cache.set_length(0, L_prev)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                gpu.cache.step(0, q, k, v, out, lse=lse, **kw)
        torch.cuda.synchronize()
        scratch = torch.empty(1 << 20, device=gpu.dev)
        for _ in range(4):
            out.zero_(); lse.zero_()
            scratch.normal_()                                  # eager work of the program's own in between
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, want) and torch.equal(lse, want_lse)
        assert gpu.cache.length(0) == L_prev + C
    finally:
        gpu.close()


@pytest.mark.parametrize("splits,upw", [(1, 1), (1, 2), (3, 1), (4, 2), (7, 1)])
def test_launch_shape_does_not_change_results_much(H, oracle, splits, upw):
    """Different launch geometries (prefix splits, rows per wave) all match the oracle."""
    cfg = I.FoldConfig("geom", 23, 1, 32, 8, 128, 192, 0, "bf16")
    chunks = [192] * 8
    outs, gpu = _fold(H, cfg, chunks, tuning={kv.TUNE_SPLITS: splits, kv.TUNE_UNITS_PER_WAVE: upw})
    oc = H.make_oracle(oracle, cfg, capacity=sum(chunks))
    pos = 0
    try:
        for step, C in enumerate(chunks):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos)
            ref, _ = H.oracle_step(oc, q, k, v, rows=[0, 1, 31, 32, 95, 190, 191])
            got = H.wide(outs[step])[[0, 1, 31, 32, 95, 190, 191]]
            assert np.abs(got - ref).max() <= 2e-2
            pos += C
    finally:
        gpu.close()


def test_resume_from_copied_rows(H):
    """The cache rows are the whole recurrent state: copy rows [0, len) into a fresh cache, set its length, go on."""
    cfg = I.FoldConfig("resume", 24, 1, 8, 2, 128, 64, 0, "bf16")
    chunks = [64] * 8
    full, g0 = _fold(H, cfg, chunks); g0.close()
    first, g1 = _fold(H, cfg, chunks[:4])
    g2 = H.GpuFold(cfg, capacity=sum(chunks), chunk_tokens=64)
    try:
        k1, v1 = g1.cache.view(0)
        k2, v2 = g2.cache.view(0)
        n = 4 * 64
        k2[:, :n].copy_(k1[:, :n]); v2[:, :n].copy_(v1[:, :n])
        torch.cuda.synchronize()
        g2.cache.set_length(0, n)
        for step in range(4, 8):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=64, token_base=step * 64)
            out = g2.step(0, q, k, v).cpu()
            assert torch.equal(out, full[step])
    finally:
        g1.close(); g2.close()


def test_rewind_and_reappend(H):
    """truncate shrinks the host-side length; re-running the step re-appends identical rows."""
    cfg = I.FoldConfig("rewind", 25, 1, 8, 2, 128, 64, 0, "bf16")
    outs, gpu = _fold(H, cfg, [64] * 4)
    try:
        assert kv.kvfold_cache_truncate(gpu.cache.handle, 0, 257) == -3   # shrink only
        assert gpu.cache.length(0) == 256
        gpu.cache.truncate(0, 128)
        assert gpu.cache.length(0) == 128
        for step in (2, 3):
            q, k, v = I.chunk_qkv(cfg, 0, step, n_tokens=64, token_base=step * 64)
            assert torch.equal(gpu.step(0, q, k, v).cpu(), outs[step])
    finally:
        gpu.close()


def test_errors_leave_the_cache_untouched(H):
    cfg = I.FoldConfig("err", 26, 2, 8, 2, 128, 64, 0, "bf16")
    gpu = H.GpuFold(cfg, capacity=128, chunk_tokens=64)
    dev = gpu.dev
    try:
        q, k, v = (t.to(dev) for t in I.chunk_qkv(cfg, 0, 0))
        out = torch.empty_like(q)
        h = gpu.cache.handle
        args = (q.data_ptr(), k.data_ptr(), v.data_ptr())
        assert kv.kvfold_step(h, 2, *args, 0, out.data_ptr(), 0) == -2          # bad layer
        assert kv.kvfold_step(h, -1, *args, 0, out.data_ptr(), 0) == -2
        assert kv.kvfold_step(h, 0, *args, 5, out.data_ptr(), 0) == -3          # position does not continue
        assert kv.kvfold_step(h, 0, None, k.data_ptr(), v.data_ptr(), 0, out.data_ptr(), 0) == -1
        assert kv.kvfold_step(h, 0, q.data_ptr() + 2, k.data_ptr(), v.data_ptr(), 0, out.data_ptr(), 0) == -1  # misaligned
        assert kv.kvfold_step_ex(h, 0, *args, 0, 0, out.data_ptr(), None, 0) == -1   # n_tokens = 0
        assert kv.kvfold_step_ex(h, 0, *args, 65, 0, out.data_ptr(), None, 0) == -1  # n_tokens > chunk_tokens
        assert kv.kvfold_cache_length(h, 0) == 0
        assert kv.kvfold_step(h, 0, *args, 0, out.data_ptr(), 0) == 0
        assert kv.kvfold_step(h, 0, *args, 64, out.data_ptr(), 0) == 0
        torch.cuda.synchronize()
        kview, _ = gpu.cache.view(0)
        before = kview.clone()
        assert kv.kvfold_step(h, 0, *args, 128, out.data_ptr(), 0) == -4        # capacity exhausted
        torch.cuda.synchronize()
        assert kv.kvfold_cache_length(h, 0) == 128 and kv.kvfold_cache_length(h, 1) == 0
        assert torch.equal(kview, before)
        assert kv.kvfold_cache_set_length(h, 0, 129) == -4
        assert kv.kvfold_cache_set_length(h, 3, 0) == -2
        assert kv.kvfold_cache_truncate(h, 3, 0) == -2 and kv.kvfold_cache_truncate(h, 0, -1) == -1
        assert kv.kvfold_cache_truncate(h, -1, 1) == -3 and kv.kvfold_cache_length(h, 0) == 128
        assert kv.kvfold_cache_truncate(h, -1, 0) == 0 and kv.kvfold_cache_length(h, 0) == 0
        assert kv.kvfold_cache_set_tuning(h, 99, 0) == -1 and kv.kvfold_cache_set_tuning(h, kv.TUNE_UNITS_PER_WAVE, 3) == -1
        assert kv.kvfold_cache_plan(h, 0, 64)[0] == -1
    finally:
        gpu.close()


def test_caller_buffer_with_guard_bands(H, oracle):
    """A caller-owned K/V buffer is used in place; bytes before and after it are never written."""
    cfg = I.FoldConfig("guard", 27, 2, 8, 2, 128, 100, 0, "bf16")
    cap = 300
    c = binding.make_config(2, 8, 2, 128, 100, cap, kv.KVFOLD_BF16)
    need = kv.kvfold_cache_bytes_required(c)
    guard = 4096
    buf = torch.full((need + 2 * guard,), 0x5A, dtype=torch.uint8, device="cuda:0")
    base = buf.data_ptr()
    off = (-base) % 256 + 256
    c.kv_buffer, c.kv_buffer_bytes = base + off, need
    rc, h = kv.kvfold_cache_create(c)
    assert rc == 0
    try:
        oc = H.make_oracle(oracle, cfg, capacity=cap)
        pos = 0
        for step, C in enumerate([100, 100, 37]):
            q, k, v = I.chunk_qkv(cfg, 1, step, n_tokens=C, token_base=pos)
            qd, kd, vd = (t.cuda() for t in (q, k, v))
            out = torch.empty_like(qd)
            assert kv.kvfold_step_ex(h, 1, qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), C, pos, out.data_ptr(), None,
                                     torch.cuda.current_stream().cuda_stream) == 0
            ref, _ = H.oracle_step(oc, q, k, v)
            torch.cuda.synchronize()
            assert np.abs(H.wide(out) - ref).max() <= 2e-2
            pos += C
        torch.cuda.synchronize()
        assert (buf[:off] == 0x5A).all() and (buf[off + need:] == 0x5A).all()
        # layer 0 was never stepped: its rows are untouched; layer 1 rows past the length too
        rc, kp, vp, rs, hs = kv.kvfold_cache_view(h, 1)
        assert rc == 0 and rs == 128 and hs == cap * 128
        k_off = kp - base
        layer_bytes = 2 * cap * 128 * 2
        assert k_off == off + layer_bytes                       # K block: [layer][head][cap][d]
        assert (buf[off:off + layer_bytes] == 0x5A).all()       # layer 0 K rows
        kl1 = buf[k_off:k_off + layer_bytes].view(torch.bfloat16).view(2, cap, 128)
        assert (kl1[:, pos:].view(torch.uint8) == 0x5A).all()   # rows past the length
        assert np.array_equal(H.bits(kl1[:, :pos]), oc.k_bits[:, :pos])
    finally:
        assert kv.kvfold_cache_destroy(h) == 0
    assert (buf[:off] == 0x5A).all()                            # destroy frees nothing of ours


def test_plan_and_profile_api(H):
    cfg = I.FoldConfig("plan", 28, 1, 32, 8, 128, 256, 0, "bf16")
    gpu = H.GpuFold(cfg, capacity=8192, chunk_tokens=256)
    try:
        wgs, splits = gpu.cache.plan(256, 8192)
        assert splits > 1 and wgs % splits == 0                # a small chunk on a long prefix is split
        gpu.cache.set_tuning(kv.TUNE_SPLITS, 1)
        assert gpu.cache.plan(256, 8192)[1] == 1
        gpu.cache.set_tuning(kv.TUNE_SPLITS, 0)
        gpu.cache.profile_begin(4)
        for step in range(6):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            gpu.step(0, q, k, v)
        n, a, t, m = gpu.cache.profile_end()
        assert n == 4 and a == 0 and t > 0 and m >= 0          # lengths are multiples of 64: the attention kernel appends
        gpu.cache.set_tuning(kv.TUNE_FUSED_APPEND, 1)
        gpu.cache.profile_begin(2)
        for step in range(6, 8):
            q, k, v = I.chunk_qkv(cfg, 0, step)
            gpu.step(0, q, k, v)
        n, a, t, m = gpu.cache.profile_end()
        assert n == 2 and a > 0 and t > 0 and m >= 0           # the append as its own kernel
    finally:
        gpu.close()


def test_binding_rejects_mismatched_tensors_before_the_library_sees_them(H):
    """The kernels trust element types and shapes, so the torch wrapper must stop a mismatch itself (a bf16 tensor
    handed to an fp32 cache, a short k_new, a host tensor) with a ValueError; nothing is enqueued, the cache stays empty."""
    cfg = I.FoldConfig("binding", 27, 1, 8, 2, 128, 64, 0, "f32")
    gpu = H.GpuFold(cfg, capacity=128, chunk_tokens=64)
    try:
        q, k, v = (t.to(gpu.dev) for t in I.chunk_qkv(cfg, 0, 0))
        out = torch.empty_like(q)
        bad = [
            (q.bfloat16(), k, v, out),                  # wrong element type
            (q, k[:32], v, out),                        # short k_new
            (q, k, v.cpu(), out),                       # host tensor
            (q, k, v, out[:, :4]),                      # wrong head count (and not contiguous)
            (q.transpose(0, 1), k, v, out),             # wrong layout
        ]
        for args in bad:
            with pytest.raises(ValueError):
                gpu.cache.step(0, *args)
        with pytest.raises(ValueError):
            gpu.cache.step(0, q, k, v, out, lse=torch.empty((8, 64), dtype=torch.float64, device=gpu.dev))
        assert gpu.cache.length(0) == 0
        gpu.cache.step(0, q, k, v, out)
        torch.cuda.synchronize()
        assert gpu.cache.length(0) == 64
    finally:
        gpu.close()


def test_measured_peaks_are_plausible(H):
    """kvfold_measure_peaks: the loop of nothing but bf16 matrix instructions lands between a third of and the whole
    datasheet rate (2516.6 TFLOP/s at 2.4 GHz; the chip clocks lower under that load), the streaming read between
    a third of and the whole 8 TB/s; either output may be left out; a bad device ordinal is refused."""
    rc, tflops, gbps = kv.kvfold_measure_peaks(0)
    assert rc == 0
    assert 800.0 < tflops < 2516.6 * 1.02, tflops
    assert 2500.0 < gbps < 8000.0, gbps
    rc, t2, g2 = kv.kvfold_measure_peaks(0, hbm=False)
    assert rc == 0 and g2 is None and abs(t2 - tflops) < 0.3 * tflops
    assert kv.kvfold_measure_peaks(-1)[0] == -1 and kv.kvfold_measure_peaks(1 << 20)[0] == -1
    print(f"box: bf16 matrix instructions only {tflops:.0f} TFLOP/s, streaming read {gbps:.0f} GB/s")
