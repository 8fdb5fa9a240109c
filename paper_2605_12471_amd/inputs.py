"""Seeded synthetic inputs for the fold step (shared by the tests, the benchmark and the smoke check).

This module only *draws numbers*: it contains none of the fold step's
arithmetic (no attention, no softmax, no cache logic) and imports neither the
HIP binding nor the CPU oracle.  The same tensors it returns are handed to both
sides of every parity comparison.

The paper runs its chains on PG-19 text through frozen Llama / Qwen models
(Sec. 2, Sec. 5 "Scaling to long contexts"); neither text nor weights are
available offline, so per-layer Q/K/V activations are replaced by i.i.d. N(0,1)
draws with the paper's shapes (Llama-3.1-8B: 32 query heads, 8 KV heads, head
dim 128 -- Tab. 4 caption; chunk sizes and chain depths of Sec. 5).
"""
from __future__ import annotations

import dataclasses
import functools
import math
import hashlib
from typing import Optional

import torch

BASE_SEED = 20260512


@dataclasses.dataclass(frozen=True)
class FoldConfig:
    """Shape of one synthetic fold workload (one entry of the benchmark's config list)."""
    name: str
    config_id: int
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    chunk: int
    total_tokens: int
    dtype: str  # "f32" | "bf16"
    needle: bool = False

    @property
    def n_steps(self) -> int:
        return self.total_tokens // self.chunk

    def with_(self, **kw) -> "FoldConfig":
        return dataclasses.replace(self, **kw)


# The five workloads of the benchmark definition.
CONFIGS = {
    "tiny_f32": FoldConfig("tiny_f32", 0, 1, 4, 1, 64, 128, 512, "f32"),
    "llama_16k": FoldConfig("llama_16k", 1, 1, 32, 8, 128, 2048, 16384, "bf16"),
    "deep_chain_128k": FoldConfig("deep_chain_128k", 2, 1, 32, 8, 128, 256, 131072, "bf16", needle=True),
    "full_stack_128k": FoldConfig("full_stack_128k", 3, 32, 32, 8, 128, 4096, 131072, "bf16"),
    "sweep_64k": FoldConfig("sweep_64k", 4, 1, 28, 4, 128, 2048, 65536, "bf16"),
}


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def _seed(*parts) -> int:
    """Counter-style seed: a stable 63-bit hash of the identifying tuple."""
    h = hashlib.sha256(repr(parts).encode()).digest()
    return int.from_bytes(h[:8], "little") & ((1 << 63) - 1)


def draw_normal(shape, dtype: torch.dtype, device, *key) -> torch.Tensor:
    """N(0,1) tensor drawn in fp32 from a generator seeded by ``key``, then cast to ``dtype``."""
    g = torch.Generator(device=device)
    g.manual_seed(_seed(BASE_SEED, *key))
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32).to(dtype)


def chunk_qkv(cfg: FoldConfig, layer: int, step: int, device="cpu", n_tokens: Optional[int] = None,
              token_base: Optional[int] = None):
    """Q [C][Hq][d], K_new [C][Hkv][d], V_new [C][Hkv][d] for chunk ``step`` of ``layer``.

    Values depend only on (config_id, layer, tensor, absolute token index range),
    NOT on the chunk size: chunk ``step`` of size C covers tokens
    [step*C, (step+1)*C) of one fixed per-layer token stream, drawn in fixed
    groups of ``_GROUP_TOKENS`` tokens.  That makes runs with different chunk sizes
    see identical token streams (needed for the chunk-size sweep).
    """
    C = cfg.chunk if n_tokens is None else n_tokens
    t0 = step * cfg.chunk if token_base is None else token_base
    dt = torch_dtype(cfg.dtype)
    out = []
    for tensor_id, heads in ((0, cfg.n_q_heads), (1, cfg.n_kv_heads), (2, cfg.n_kv_heads)):
        out.append(_token_range(cfg, layer, tensor_id, heads, t0, t0 + C, dt, device))
    q, k, v = out
    if cfg.needle:
        spec = needle_spec(cfg)
        if t0 <= spec.key_pos < t0 + C:
            k = plant_needle_key(cfg, k, t0, device)
    return q, k, v


_GROUP_TOKENS = 4096  # tokens per generator call; fixed, so streams do not depend on the chunk size


@functools.lru_cache(maxsize=6)
def _token_group(config_id, layer, tensor_id, heads, head_dim, dt, device, gidx):
    return draw_normal((_GROUP_TOKENS, heads, head_dim), dt, device, config_id, layer, tensor_id, gidx)


def _token_range(cfg, layer, tensor_id, heads, t_lo, t_hi, dt, device):
    """Tokens [t_lo, t_hi) of the fixed per-(layer, tensor) stream, drawn in groups of _GROUP_TOKENS."""
    parts = []
    for gidx in range(t_lo // _GROUP_TOKENS, (t_hi + _GROUP_TOKENS - 1) // _GROUP_TOKENS):
        blk = _token_group(cfg.config_id, layer, tensor_id, heads, cfg.head_dim, dt, str(device), gidx)
        lo = max(t_lo, gidx * _GROUP_TOKENS) - gidx * _GROUP_TOKENS
        hi = min(t_hi, (gidx + 1) * _GROUP_TOKENS) - gidx * _GROUP_TOKENS
        parts.append(blk[lo:hi])
    return parts[0].contiguous().clone() if len(parts) == 1 else torch.cat(parts, 0).contiguous()


LOGIT_PROFILES = {
    # logit (in nats, up to the noise) of every query against key j, as a function of the absolute key index
    "step20": lambda j: 20.0 * (j >= 100),     # one jump of 20 nats inside the prefix
    "step45": lambda j: 45.0 * (j >= 100),     # ... of 45 nats (2^65 in one go)
    "step100": lambda j: 100.0 * (j >= 100),   # ... of 100 nats: exp2 of the jump overflows fp32
    "stairs": lambda j: 0.5 * j,               # rises by 16 nats every 32 keys, for ever
    "spike": lambda j: 60.0 * (j == 130),      # one dominating key, then back to the floor
    "late": lambda j: 80.0 * (j >= 290),       # the jump lies inside the causal part of the last chunk
    "deep_start": lambda j: -150.0 * (j < 96),  # the first keys lie 2^216 below the rest: a first reference far below zero
}


def steered_qkv(cfg: FoldConfig, layer: int, step: int, profile: str, device="cpu", n_tokens: Optional[int] = None,
                token_base: Optional[int] = None):
    """The stream of chunk_qkv scaled to 0.1, plus a component along one seeded unit direction u that
    gives every query the logit LOGIT_PROFILES[profile](j) against key j (softmax scale 1/sqrt(d)):
    q += 2 sqrt(d) u, k_j += (g_j / 2) u.  Stress input for the running-max bookkeeping of a kernel;
    V is the plain stream."""
    C = cfg.chunk if n_tokens is None else n_tokens
    t0 = step * cfg.chunk if token_base is None else token_base
    q, k, v = chunk_qkv(cfg.with_(needle=False) if cfg.needle else cfg, layer, step, device, n_tokens, token_base)
    d = cfg.head_dim
    u = draw_normal((d,), torch.float32, device, cfg.config_id, layer, 9)
    u = u / u.norm()
    g = torch.tensor([LOGIT_PROFILES[profile](j) for j in range(t0, t0 + C)], dtype=torch.float32, device=device)
    dt = torch_dtype(cfg.dtype)
    q = (0.1 * q.float() + 2.0 * math.sqrt(d) * u).to(dt)
    k = (0.1 * k.float() + 0.5 * g[:, None, None] * u).to(dt)
    return q, k, v


def rope_tables(head_dim: int, pos0: int, n_tokens: int, theta: float = 500000.0, device="cpu"):
    """cos / sin [n_tokens][head_dim/2] fp32 of the angles (pos0 + i) * theta^(-2j/head_dim): what a model's
    rotary cache holds for the absolute positions of one chunk (theta = 500000 is the Llama-3 base).
    Angles are formed in fp64 and rounded once."""
    j = torch.arange(head_dim // 2, dtype=torch.float64)
    inv_freq = theta ** (-2.0 * j / head_dim)
    ang = torch.arange(pos0, pos0 + n_tokens, dtype=torch.float64)[:, None] * inv_freq[None, :]
    return ang.cos().float().to(device).contiguous(), ang.sin().float().to(device).contiguous()


@dataclasses.dataclass(frozen=True)
class NeedleSpec:
    key_pos: int      # absolute token position of the planted key (inside chunk 0)
    query_row: int    # absolute token position of the probing query (inside the last chunk)
    query_head: int   # query head of the probing row
    gain: float       # planted key = gain * q / ||q||


def needle_spec(cfg: FoldConfig) -> NeedleSpec:
    g = torch.Generator(device="cpu")
    g.manual_seed(_seed(BASE_SEED, cfg.config_id, "needle"))
    r = torch.randint(0, 1 << 30, (3,), generator=g).tolist()
    key_pos = r[0] % cfg.chunk
    query_row = cfg.total_tokens - cfg.chunk + (r[1] % cfg.chunk)
    return NeedleSpec(key_pos, query_row, r[2] % cfg.n_q_heads, 8.0)


def plant_needle_key(cfg: FoldConfig, k_chunk: torch.Tensor, t0: int, device) -> torch.Tensor:
    """Overwrite the needle's key row (KV head of the probing query head) with gain * q / ||q||."""
    spec = needle_spec(cfg)
    dt = torch_dtype(cfg.dtype)
    q_row = _token_range(cfg.with_(needle=False), 0, 0, cfg.n_q_heads, spec.query_row, spec.query_row + 1,
                         dt, device)[0, spec.query_head].float()
    key = (spec.gain * q_row / q_row.norm()).to(dt)
    k_chunk = k_chunk.clone()
    k_chunk[spec.key_pos - t0, spec.query_head // (cfg.n_q_heads // cfg.n_kv_heads)] = key
    return k_chunk


def sample_steps(cfg: FoldConfig, n_random: int = 8):
    """Chain steps on which sampled parity is checked: both ends, the middle, plus seeded random ones."""
    N = cfg.n_steps
    fixed = {0, 1, 2, N // 2, N - 2, N - 1}
    g = torch.Generator(device="cpu")
    g.manual_seed(_seed(BASE_SEED, cfg.config_id, "sample_steps"))
    rnd = set(torch.randint(0, N, (n_random,), generator=g).tolist())
    return sorted(s for s in (fixed | rnd) if 0 <= s < N)


def sample_rows(cfg: FoldConfig, step: int, n_random: int = 16, C: Optional[int] = None):
    """Chunk rows on which sampled parity is checked at ``step``."""
    C = cfg.chunk if C is None else C
    fixed = {0, 1, C // 2, C - 2, C - 1}
    g = torch.Generator(device="cpu")
    g.manual_seed(_seed(BASE_SEED, cfg.config_id, "sample_rows", step))
    rnd = set(torch.randint(0, C, (n_random,), generator=g).tolist())
    return sorted(r for r in (fixed | rnd) if 0 <= r < C)
