"""kvfold_step_noalloc (the entry point for callers that cannot allocate: split partials in a static device
array) against kvfold_step_ex, through the C ABI: two calls in a row on one GPU, the second with a smaller
input, on shapes whose key range is split (so the scratch array is really used), plus an unsplit one and the
size limit."""
import numpy as np
import pytest
import torch

import paper_2605_12471_amd as kv
from paper_2605_12471_amd import inputs as I

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _filled_cache(cfg, C, L_prev, cap, seed):
    cache = kv.KvFoldCache(1, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, C, cap, cfg.dtype)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    K, V = cache.view(0)
    K[:, :L_prev].normal_(generator=g)
    V[:, :L_prev].normal_(generator=g)
    cache.set_length(0, L_prev)
    return cache


@pytest.mark.parametrize("dtype,tol", [("bf16", 2e-2), ("f32", 1e-5)])
def test_noalloc_step_matches_step_ex_on_two_calls_in_a_row(dtype, tol):
    cfg = I.FoldConfig("noalloc", 60, 1, 8, 2, 128, 64, 0, dtype)
    cap = 8192
    # first call: 64 rows against 8000 keys; second call: 16 rows (smaller input) against 4000 keys
    results = {}
    for which in ("ex", "noalloc"):
        outs = []
        for C, L_prev, seed in ((64, 8000, 1), (16, 4000, 2)):
            cache = _filled_cache(cfg, 64, L_prev, cap, seed)
            assert cache.plan(C, L_prev + C)[1] > 1, "the key range must be split for the scratch array to be used"
            q, k, v = (t.to(DEV) for t in I.chunk_qkv(cfg, 0, seed, n_tokens=C, token_base=L_prev))
            out = torch.empty_like(q)
            lse = torch.empty((cfg.n_q_heads, C), dtype=torch.float32, device=DEV)
            fn = kv.kvfold_step_ex if which == "ex" else kv.kvfold_step_noalloc
            rc = fn(cache.handle, 0, q.data_ptr(), k.data_ptr(), v.data_ptr(), C, L_prev, out.data_ptr(), lse.data_ptr(),
                    torch.cuda.current_stream().cuda_stream)
            assert rc == 0, kv.kvfold_status_string(rc)
            torch.cuda.synchronize()
            Kc, Vc = cache.view(0)
            outs.append((out.float().cpu(), lse.cpu(), Kc[:, L_prev:L_prev + C].clone().cpu(), Vc[:, L_prev:L_prev + C].clone().cpu()))
            cache.close()
        results[which] = outs
    for (o1, l1, k1, v1), (o2, l2, k2, v2) in zip(results["ex"], results["noalloc"]):
        assert float((o1 - o2).abs().max()) <= tol
        assert float((l1 - l2).abs().max()) <= (2e-2 if dtype == "bf16" else 1e-5)
        assert torch.equal(k1.view(torch.int16 if dtype == "bf16" else torch.int32), k2.view(torch.int16 if dtype == "bf16" else torch.int32))
        assert torch.equal(v1.view(torch.int16 if dtype == "bf16" else torch.int32), v2.view(torch.int16 if dtype == "bf16" else torch.int32))


def test_noalloc_interleaved_on_one_cache_and_unsplit():
    """Both entry points alternate on one cache (stream-ordered): a deep chain of C = 256 steps (8 splits), bit-equal
    when both plans agree; then a chunk too long to need a split (no scratch use at all)."""
    cfg = I.FoldConfig("noalloc_chain", 61, 1, 32, 8, 128, 256, 0, "bf16")
    cap = 32768
    a = _filled_cache(cfg, 256, 30000 - 30000 % 64, cap, 3)
    b = _filled_cache(cfg, 256, 30000 - 30000 % 64, cap, 3)
    try:
        pos = a.length(0)
        for step in range(4):
            C = 256 if step != 2 else 100           # the third call is smaller
            q, k, v = (t.to(DEV) for t in I.chunk_qkv(cfg, 0, step, n_tokens=C, token_base=pos))
            oa, ob = torch.empty_like(q), torch.empty_like(q)
            a.step(0, q, k, v, oa)
            b.step(0, q, k, v, ob, noalloc=True)
            torch.cuda.synchronize()
            assert float((oa.float() - ob.float()).abs().max()) <= 2e-2
            pos += C
        Ka, Va = a.view(0)
        Kb, Vb = b.view(0)
        assert torch.equal(Ka[:, :pos], Kb[:, :pos]) and torch.equal(Va[:, :pos], Vb[:, :pos])
    finally:
        a.close()
        b.close()


def test_noalloc_rejects_steps_beyond_the_scratch_array():
    """n_tokens * n_q_heads above 65536 rows cannot place two pieces in the array: KVFOLD_ERR_SCRATCH, nothing
    enqueued, the cache untouched."""
    cfg = I.FoldConfig("noalloc_big", 62, 1, 32, 8, 128, 4096, 0, "bf16")
    cache = kv.KvFoldCache(1, 32, 8, 128, 4096, 8192, "bf16")
    try:
        q, k, v = (t.to(DEV) for t in I.chunk_qkv(cfg, 0, 0))
        out = torch.empty_like(q)
        rc = kv.kvfold_step_noalloc(cache.handle, 0, q.data_ptr(), k.data_ptr(), v.data_ptr(), 4096, 0, out.data_ptr(), None, 0)
        assert rc == -8 and kv.kvfold_status_string(rc).startswith("step does not fit")
        assert cache.length(0) == 0
        # 2048 rows x 32 heads = 65536 rows: the largest step that fits
        rc = kv.kvfold_step_noalloc(cache.handle, 0, q.data_ptr(), k.data_ptr(), v.data_ptr(), 2048, 0, out.data_ptr(), None, 0)
        assert rc == 0
        torch.cuda.synchronize()
        assert cache.length(0) == 2048
    finally:
        cache.close()


def test_noalloc_step_under_graph_capture():
    """The callers this entry point is for: a split step (64 pieces + merge, partials in the static array) captured into
    a HIP graph and replayed several times, with eager work and synchronisations between the replays, gives the bits
    of the eager call."""
    cfg = I.FoldConfig("noalloc_graph", 63, 1, 8, 2, 128, 16, 0, "bf16")
    C, L_prev = 16, 6000
    cache = _filled_cache(cfg, 16, L_prev, 8192, 5)
    try:
        assert cache.plan(C, L_prev + C)[1] > 1
        q, k, v = (t.to(DEV) for t in I.chunk_qkv(cfg, 0, 7, n_tokens=C, token_base=L_prev))
        out = torch.empty_like(q)
        lse = torch.empty((cfg.n_q_heads, C), dtype=torch.float32, device=DEV)
        cache.step(0, q, k, v, out, lse=lse, noalloc=True)
        torch.cuda.synchronize()
        want, want_lse = out.clone(), lse.clone()
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        cache.set_length(0, L_prev)
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                cache.step(0, q, k, v, out, lse=lse, noalloc=True)
        torch.cuda.synchronize()
        scratch = torch.empty(1 << 20, device=DEV)
        for _ in range(4):
            out.zero_(); lse.zero_()
            scratch.normal_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, want) and torch.equal(lse, want_lse)
        assert cache.length(0) == L_prev + C
    finally:
        cache.close()
