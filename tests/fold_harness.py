"""Shared helpers of the GPU parity tests: run a fold through the C-ABI library and through the oracle
on the same seeded tensors.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

import paper_2605_12471_amd as kv
from paper_2605_12471_amd import inputs as I

TOL = {"f32": 1e-5, "bf16": 2e-2}   # max-abs tolerances of the benchmark definition


def bits(t: torch.Tensor) -> np.ndarray:
    """Raw stored element bits of a CPU tensor as numpy (uint16 for bf16, float32 for f32)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def wide(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().double().numpy()


class GpuFold:
    """One library cache + output buffers for a FoldConfig."""

    def __init__(self, cfg: I.FoldConfig, capacity=None, chunk_tokens=None, n_layers=None, device="cuda:0"):
        self.cfg = cfg
        self.dev = torch.device(device)
        self.cache = kv.KvFoldCache(n_layers or cfg.n_layers, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                                    chunk_tokens or cfg.chunk, capacity or cfg.total_tokens, cfg.dtype,
                                    device=self.dev.index or 0)

    def step(self, layer, q, k, v, want_lse=False, rope=None, window=None, noalloc=False):
        q, k, v = (t.to(self.dev).contiguous() for t in (q, k, v))
        out = torch.empty_like(q)
        lse = torch.empty((self.cfg.n_q_heads, q.shape[0]), dtype=torch.float32, device=self.dev) if want_lse else None
        if rope is not None:
            rope = tuple(t.to(self.dev).contiguous() for t in rope)
        self.cache.step(layer, q, k, v, out, lse=lse, rope=rope, window=window, noalloc=noalloc)
        return (out, lse) if want_lse else out

    def close(self):
        self.cache.close()


def make_oracle(oracle_mod, cfg: I.FoldConfig, capacity=None):
    store = np.uint16 if cfg.dtype == "bf16" else np.float32
    return oracle_mod.OracleCache(cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, capacity or cfg.total_tokens,
                                  store_dtype=store)


def oracle_step(ocache, q, k, v, rows=None, want_weights=False, window=None):
    """q/k/v are the torch tensors handed to the GPU (CPU copies); K/V stored bit-exactly, q widened.
    window = (n_sink, window): the sink + sliding-window step."""
    n_sink, win = window if window is not None else (0, None)
    return ocache.step(wide(q), bits(k), bits(v), ocache.len, rows=rows, want_weights=want_weights,
                       n_sink=n_sink, window=win)


def assert_cache_bit_exact(gpu: GpuFold, ocache, layer=0):
    kd, vd = gpu.cache.view(layer)
    n = ocache.len
    assert gpu.cache.length(layer) == n
    torch.cuda.synchronize()
    assert np.array_equal(bits(kd[:, :n]), ocache.k_bits[:, :n]), "K cache differs from the appended rows"
    assert np.array_equal(bits(vd[:, :n]), ocache.v_bits[:, :n]), "V cache differs from the appended rows"
