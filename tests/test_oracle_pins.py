"""Pins for the fp64 CPU oracle: what the paper and the mathematics fix, none of it the oracle's own code.

* fold invariant (Sec. 2: keys K_{0:t} are the concatenation of all chunks and positions continue,
  so any chunking must reproduce the FULL condition's single causal pass),
* brute-force python loops on tiny inputs,
* torch's fp64 scaled_dot_product_attention as an independent library routine,
* closed forms and invariances of softmax attention,
* the planted-needle weight in closed form.
"""
import math

import numpy as np
import pytest
import torch


def _rand(T, Hq, Hkv, d, seed):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((T, Hq, d)), rng.standard_normal((T, Hkv, d)), rng.standard_normal((T, Hkv, d)))


def _brute(Q, K, V, scale):
    """Pure python triple loop: the definition with nothing vectorised."""
    T, Hq, d = Q.shape
    G = Hq // K.shape[1]
    out = np.zeros((T, Hq, d))
    for i in range(T):
        for h in range(Hq):
            g = h // G
            s = [scale * sum(Q[i, h, x] * K[j, g, x] for x in range(d)) for j in range(i + 1)]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            l = sum(e)
            for j in range(i + 1):
                for x in range(d):
                    out[i, h, x] += e[j] / l * V[j, g, x]
    return out


@pytest.mark.parametrize("Hq,Hkv,d", [(4, 1, 8), (4, 2, 8), (4, 4, 16), (6, 3, 8)])
def test_brute_force_tiny(oracle, Hq, Hkv, d):
    T = 12
    Q, K, V = _rand(T, Hq, Hkv, d, 1)
    ref = _brute(Q, K, V, 1 / math.sqrt(d))
    for chunks in ([T], [1] * T, [5, 7], [3, 3, 3, 3], [1, 11]):
        out, _ = oracle.fold(Q, K, V, chunks)
        assert np.abs(out - ref).max() < 1e-13, chunks
    mono, _ = oracle.monolithic_causal_attention(Q, K, V)
    assert np.abs(mono - ref).max() < 1e-13


@pytest.mark.parametrize("T,Hq,Hkv,d", [(64, 4, 1, 8), (192, 4, 2, 64), (512, 4, 1, 64), (200, 8, 4, 32)])
def test_fold_invariant_vs_monolithic(oracle, T, Hq, Hkv, d):
    Q, K, V = _rand(T, Hq, Hkv, d, 2)
    mono, mono_lse = oracle.monolithic_causal_attention(Q, K, V)
    chunkings = [[T], [1] * T, [T // 2, T - T // 2], [7] * (T // 7) + ([T % 7] if T % 7 else []),
                 [3] * (T // 3) + ([T % 3] if T % 3 else []), [T - 1, 1], [1, T - 1]]
    if T % 128 == 0:
        chunkings.append([128] * (T // 128))
    for chunks in chunkings:
        out, lse = oracle.fold(Q, K, V, chunks)
        assert np.abs(out - mono).max() < 1e-12
        assert np.abs(lse - mono_lse).max() < 1e-12


def test_chunk_size_independence(oracle):
    T = 256
    Q, K, V = _rand(T, 4, 2, 16, 3)
    outs = [oracle.fold(Q, K, V, [C] * (T // C))[0] for C in (1, 8, 32, 128, 256)]
    for o in outs[1:]:
        assert np.abs(o - outs[0]).max() < 1e-12


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 2), (28, 4)])
def test_vs_torch_sdpa_fp64(oracle, Hq, Hkv):
    T, d = 96, 32
    Q, K, V = _rand(T, Hq, Hkv, d, 4)
    G = Hq // Hkv
    tq = torch.from_numpy(Q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    out, _ = oracle.fold(Q, K, V, [32, 32, 32])
    assert np.abs(out - ref).max() < 1e-12


def test_prefix_visible_causal_inside_chunk(oracle):
    """Step with a non-empty prefix vs torch SDPA with an explicit boolean mask (prefix visible + causal)."""
    Lp, C, Hq, Hkv, d = 40, 24, 4, 2, 16
    Q, K, V = _rand(Lp + C, Hq, Hkv, d, 5)
    cache = oracle.OracleCache(Hq, Hkv, d, Lp + C)
    cache.append(K[:Lp], V[:Lp])
    out, _ = cache.step(Q[Lp:], K[Lp:], V[Lp:], Lp)
    mask = torch.zeros(C, Lp + C, dtype=torch.bool)
    for i in range(C):
        mask[i, : Lp + i + 1] = True
    tq = torch.from_numpy(Q[Lp:]).permute(1, 0, 2)[None]
    tk = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    tv = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(2, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    assert np.abs(out - ref).max() < 1e-12


def test_weights_rows_sum_to_one_and_respect_mask(oracle):
    Lp, C, Hq, Hkv, d = 10, 6, 4, 2, 8
    Q, K, V = _rand(Lp + C, Hq, Hkv, d, 6)
    cache = oracle.OracleCache(Hq, Hkv, d, Lp + C)
    cache.append(K[:Lp], V[:Lp])
    out, lse, w = cache.step(Q[Lp:], K[Lp:], V[Lp:], Lp, want_weights=True)
    assert np.abs(w.sum(-1) - 1).max() < 1e-14
    for i in range(C):
        assert (w[i, :, Lp + i + 1:] == 0).all()      # future keys carry no weight
        assert (w[i, :, : Lp + i + 1] > 0).all()      # every visible key carries some
    # out is the weight-average of the visible value rows (convex hull, componentwise bound)
    for i in range(C):
        for h in range(Hq):
            vis = V[: Lp + i + 1, h // 2]
            assert (out[i, h] <= vis.max(0) + 1e-12).all() and (out[i, h] >= vis.min(0) - 1e-12).all()
            assert np.abs(out[i, h] - w[i, h, : Lp + i + 1] @ vis).max() < 1e-13
    # lse is the log of the unnormalised mass: weights == exp(logit - lse)
    s = np.einsum("chd,jhd->chj", Q[Lp:], np.repeat(K, 2, 1)) / math.sqrt(d)
    for i in range(C):
        n = Lp + i + 1
        assert np.abs(np.exp(s[i, :, :n] - lse[i][:, None]) - w[i, :, :n]).max() < 1e-13


def test_first_row_and_single_key(oracle):
    Q, K, V = _rand(5, 4, 2, 8, 7)
    out, lse = oracle.fold(Q, K, V, [5])
    for h in range(4):
        assert np.array_equal(out[0, h], V[0, h // 2])  # one visible key: out is that value row exactly
        assert abs(lse[0, h] - (Q[0, h] @ K[0, h // 2]) / math.sqrt(8)) < 1e-14


def test_closed_forms(oracle):
    T, Hq, Hkv, d = 33, 4, 2, 8
    Q, K, V = _rand(T, Hq, Hkv, d, 8)
    # all keys equal -> uniform weights -> running mean of V
    Keq = np.broadcast_to(K[:1], K.shape).copy()
    out, _ = oracle.fold(Q, Keq, V, [11, 22])
    for i in range(T):
        for h in range(Hq):
            assert np.abs(out[i, h] - V[: i + 1, h // 2].mean(0)).max() < 1e-13
    # constant V -> out is that constant
    Vc = np.broadcast_to(V[:1], V.shape).copy()
    out, _ = oracle.fold(Q, K, Vc, [10, 23])
    assert np.abs(out - np.repeat(Vc, 2, 1)).max() < 1e-13
    # adding one vector c to every key shifts every logit of a row equally -> out unchanged
    c = np.random.default_rng(0).standard_normal((1, Hkv, d))
    base, base_lse = oracle.fold(Q, K, V, [T])
    shifted, shifted_lse = oracle.fold(Q, K + c, V, [T])
    assert np.abs(base - shifted).max() < 1e-12
    # ... while lse moves by exactly scale * q.c
    shift = np.einsum("thd,hd->th", Q, np.repeat(c[0], 2, 0)) / math.sqrt(d)
    assert np.abs(shifted_lse - base_lse - shift).max() < 1e-12


def test_prefix_permutation_invariance(oracle):
    Lp, C, Hq, Hkv, d = 50, 8, 4, 1, 16
    Q, K, V = _rand(Lp + C, Hq, Hkv, d, 9)
    perm = np.random.default_rng(1).permutation(Lp)

    def run(Kp, Vp):
        cache = oracle.OracleCache(Hq, Hkv, d, Lp + C)
        cache.append(Kp, Vp)
        return cache.step(Q[Lp:], K[Lp:], V[Lp:], Lp)[0]

    assert np.abs(run(K[:Lp], V[:Lp]) - run(K[:Lp][perm], V[:Lp][perm])).max() < 1e-13


def test_gqa_mapping_is_contiguous_groups(oracle):
    """Perturbing KV head g changes exactly query heads g*G .. g*G+G-1."""
    T, Hq, Hkv, d = 16, 6, 3, 8
    Q, K, V = _rand(T, Hq, Hkv, d, 10)
    base, _ = oracle.fold(Q, K, V, [T])
    V2 = V.copy()
    V2[:, 1] += 1.0
    pert, _ = oracle.fold(Q, K, V2, [T])
    changed = [h for h in range(Hq) if np.abs(pert[:, h] - base[:, h]).max() > 0]
    assert changed == [2, 3]
    assert np.abs(pert[:, 2:4] - base[:, 2:4] - 1.0).max() < 1e-12  # weights sum to 1


def test_causality_future_keys_invisible(oracle):
    T, Hq, Hkv, d = 20, 2, 1, 8
    Q, K, V = _rand(T, Hq, Hkv, d, 11)
    base, _ = oracle.fold(Q, K, V, [8, 12])
    K2, V2 = K.copy(), V.copy()
    K2[13] += 5
    V2[13] -= 3
    pert, _ = oracle.fold(Q, K2, V2, [8, 12])
    assert np.array_equal(pert[:13], base[:13])
    assert np.abs(pert[13:] - base[13:]).max() > 1e-3


def test_planted_needle_weight_closed_form(oracle):
    """One key with logit a among n-1 keys of logit 0: weight = e^a / (e^a + n - 1)."""
    n, d = 500, 16
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 4.0
    K = np.zeros((n, 1, d)); K[123, 0, 0] = 2.0           # logit = 4*2/sqrt(16) = 2
    V = np.random.default_rng(2).standard_normal((n, 1, d))
    cache = oracle.OracleCache(1, 1, d, n)
    cache.append(K[:-1], V[:-1])
    out, lse, w = cache.step(q, K[-1:], V[-1:], n - 1, want_weights=True)
    expect = math.exp(2) / (math.exp(2) + n - 1)
    assert abs(w[0, 0, 123] - expect) < 1e-15
    assert abs(lse[0, 0] - math.log(math.exp(2) + n - 1)) < 1e-13
    assert int(w[0, 0].argmax()) == 123


def test_cache_is_concatenation_of_inputs_bitwise(oracle):
    rng = np.random.default_rng(3)
    Hkv, d = 2, 8
    bits_k = rng.integers(0, 1 << 16, (30, Hkv, d), dtype=np.uint16)  # arbitrary bf16 patterns incl. NaNs
    bits_v = rng.integers(0, 1 << 16, (30, Hkv, d), dtype=np.uint16)
    cache = oracle.OracleCache(4, Hkv, d, 40, store_dtype=np.uint16)
    pos = 0
    for C in (7, 1, 22):
        cache.append(bits_k[pos:pos + C], bits_v[pos:pos + C])
        pos += C
    assert cache.len == 30
    assert np.array_equal(cache.k_bits[:, :30], bits_k.transpose(1, 0, 2))
    assert np.array_equal(cache.v_bits[:, :30], bits_v.transpose(1, 0, 2))
    assert (cache.k_bits[:, 30:] == 0).all()
    # widening of bf16 bits is exact: compare against torch's bfloat16 -> float64
    t = torch.from_numpy(bits_k.view(np.int16)).view(torch.bfloat16).double().numpy().transpose(1, 0, 2)
    finite = np.isfinite(t)
    assert np.array_equal(cache.K[:, :30][finite], t[finite])


def test_step_rejects_wrong_position_and_overflow(oracle):
    cache = oracle.OracleCache(2, 1, 4, 8)
    z = np.zeros((4, 1, 4)); q = np.zeros((4, 2, 4))
    with pytest.raises(ValueError):
        cache.step(q, z, z, 3)
    cache.step(q, z, z, 0)
    cache.step(q, z, z, 4)
    with pytest.raises(ValueError):
        cache.step(q, z, z, 8)


def test_row_subset_matches_full(oracle):
    Lp, C = 17, 9
    Q, K, V = _rand(Lp + C, 4, 2, 8, 12)
    c1 = oracle.OracleCache(4, 2, 8, Lp + C); c1.append(K[:Lp], V[:Lp])
    full, full_lse = c1.step(Q[Lp:], K[Lp:], V[Lp:], Lp)
    c2 = oracle.OracleCache(4, 2, 8, Lp + C); c2.append(K[:Lp], V[:Lp])
    sub, sub_lse = c2.step(Q[Lp:], K[Lp:], V[Lp:], Lp, rows=[0, 4, 8])
    assert np.array_equal(sub, full[[0, 4, 8]]) and np.array_equal(sub_lse, full_lse[[0, 4, 8]])


def test_pins_catch_planted_mistakes(oracle):
    """Plausible slips, planted in a copy of the definition on the CPU, must all be told apart from the oracle."""
    T, Hq, Hkv, d = 24, 4, 2, 8
    Q, K, V = _rand(T, Hq, Hkv, d, 13)
    good, _ = oracle.fold(Q, K, V, [10, 14])

    def variant(mask_k=1, head_map=lambda h: h // 2, scale=1 / math.sqrt(d), transpose_v=False):
        out = np.zeros((T, Hq, d))
        for h in range(Hq):
            g = head_map(h)
            S = (Q[:, h] @ K[:, g].T) * scale
            S[np.triu(np.ones((T, T), bool), k=mask_k)] = -np.inf
            S[:, 0] = np.where(np.isinf(S[:, 0]), 0.0, S[:, 0])  # keep rows non-empty for the strict mask
            P = np.exp(S - S.max(1, keepdims=True))
            P /= P.sum(1, keepdims=True)
            out[:, h] = P @ (V[:, g][:, ::-1] if transpose_v else V[:, g])
        return out

    assert np.abs(variant() - good).max() < 1e-12                       # the faithful copy agrees
    assert np.abs(variant(mask_k=0) - good).max() > 1e-3                # diagonal excluded
    assert np.abs(variant(mask_k=2) - good).max() > 1e-3                # one future key leaks
    assert np.abs(variant(head_map=lambda h: h % 2) - good).max() > 1e-3  # interleaved GQA mapping
    assert np.abs(variant(scale=1.0) - good).max() > 1e-3               # dropped 1/sqrt(d)
    assert np.abs(variant(transpose_v=True) - good).max() > 1e-3        # value columns reversed


def test_steered_inputs_have_the_stated_logits():
    """The stress generator of the GPU tests: q . k_j / sqrt(d) equals the profile's logit up to the 0.1-scaled
    noise (under a nat, growing with the logit through the cross term) and bf16 rounding."""
    from paper_2605_12471_amd import inputs as I
    cfg = I.FoldConfig("jumps", 15, 1, 8, 2, 128, 256, 0, "bf16")
    for profile, fn in I.LOGIT_PROFILES.items():
        q, k, _ = I.steered_qkv(cfg, 0, 0, profile)
        s = np.einsum("ihx,jgx->ihgj", q.double().numpy(), k.double().numpy()) / np.sqrt(128.0)
        want = np.array([fn(j) for j in range(256)])
        assert np.abs(s - want[None, None, None, :]).max() < 0.8 + 0.02 * np.abs(want).max(), profile


# ---- rotary embedding of the new tokens at absolute positions (Sec. 2: positions continue from tC)

def _angles(rows, hd, seed, pos0=0):
    rng = np.random.default_rng(seed)
    inv = 10000.0 ** (-np.arange(hd) / hd)
    ang = (pos0 + np.arange(rows))[:, None] * inv[None, :]
    return ang, rng


def test_rope_is_a_complex_rotation_of_the_half_split_pairs(oracle):
    """Element j and j + d/2 form the complex number x_j + i x_{j+d/2}; the rotation is multiplication by
    e^{i angle}.  Checked against numpy's complex128 arithmetic (an independent formula) to fp32 accuracy."""
    rows, heads, d = 37, 3, 64
    ang, rng = _angles(rows, d // 2, 1, pos0=1000)
    x = rng.standard_normal((rows, heads, d)).astype(np.float32)
    got = oracle.rope(x, np.cos(ang), np.sin(ang)).astype(np.float64)
    z = (x[..., : d // 2] + 1j * x[..., d // 2:]) * np.exp(1j * ang)[:, None, :]
    want = np.concatenate([z.real, z.imag], axis=-1)
    assert np.abs(got - want).max() < 5e-7 * np.abs(x).max() * 2


def test_rope_special_angles_are_exact(oracle):
    rows, heads, d = 5, 2, 16
    rng = np.random.default_rng(2)
    x = rng.standard_normal((rows, heads, d)).astype(np.float32)
    one, zero = np.ones((rows, d // 2), np.float32), np.zeros((rows, d // 2), np.float32)
    assert np.array_equal(oracle.rope(x, one, zero), x)                       # angle 0: identity (position 0)
    quarter = oracle.rope(x, zero, one)                                       # angle pi/2: (a, b) -> (-b, a)
    assert np.array_equal(quarter[..., : d // 2], -x[..., d // 2:]) and np.array_equal(quarter[..., d // 2:], x[..., : d // 2])
    assert np.array_equal(oracle.rope(x, -one, zero), -x)                     # angle pi


def test_rope_keeps_norms_and_makes_logits_depend_on_relative_position(oracle):
    """|R x| = |x|, and (R_m q).(R_n k) = (R_{m-n} q).k: the property that makes continued absolute
    positions across chunk boundaries equivalent to one long sequence."""
    heads, d = 2, 64
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, heads, d)).astype(np.float32)
    k = rng.standard_normal((1, heads, d)).astype(np.float32)
    inv = 10000.0 ** (-np.arange(d // 2) / (d // 2))

    def rot(x, pos):
        a = (pos * inv)[None, :]
        return oracle.rope(x, np.cos(a), np.sin(a)).astype(np.float64)

    for m, n in ((5, 3), (4099, 4096), (131071, 131000), (17, 17)):
        qm, kn = rot(q, m), rot(k, n)
        assert abs(np.linalg.norm(qm) - np.linalg.norm(q.astype(np.float64))) < 1e-5
        lhs = (qm * kn).sum(-1)
        rhs = (rot(q, m - n) * k.astype(np.float64)).sum(-1)
        assert np.abs(lhs - rhs).max() < 2e-4, (m, n)


def test_bf16_rounding_helper_is_round_to_nearest_even(oracle):
    """f32_to_bf16_bits against torch's own conversion on random values, ties and the largest finite value."""
    import torch
    rng = np.random.default_rng(4)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 20000),
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, -0.0, 3.3895314e38, np.inf, -np.inf], np.float32)])
    want = torch.from_numpy(x).bfloat16().view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f32_to_bf16_bits(x), want)
    assert np.array_equal(oracle.bf16_bits_to_f32(want), torch.from_numpy(x).bfloat16().float().numpy())


def test_rope_tables_generator_matches_its_formula():
    from paper_2605_12471_amd import inputs as I
    cos, sin = I.rope_tables(8, 100, 3, theta=10000.0)
    ang = np.arange(100, 103)[:, None] * 10000.0 ** (-2.0 * np.arange(4) / 8)[None, :]
    assert np.allclose(cos.numpy(), np.cos(ang), atol=1e-7) and np.allclose(sin.numpy(), np.sin(ang), atol=1e-7)


# ---- storage round trip bf16 -> intN -> bf16 of rows joining the cache (Sec. 8, Discussion)

@pytest.mark.parametrize("n_bits", [8, 4])
def test_storage_roundtrip_properties(oracle, n_bits):
    rng = np.random.default_rng(5)
    x = rng.standard_normal((200, 3, 128)).astype(np.float32) * rng.uniform(0.01, 30.0, (200, 3, 1)).astype(np.float32)
    x[7] = 0.0
    b = oracle.f32_to_bf16_bits(x)
    xb = oracle.bf16_bits_to_f32(b).astype(np.float64)
    y = oracle.bf16_bits_to_f32(oracle.storage_roundtrip(b, n_bits)).astype(np.float64)
    qmax = 2 ** (n_bits - 1) - 1
    amax = np.abs(xb).max(-1, keepdims=True)
    step = amax / qmax
    assert np.all(y[7] == 0.0)                                                    # zero row stays zero
    assert np.all(np.abs(y - xb) <= step / 2 * 1.0001 + np.abs(y) * 2.0 ** -8)      # half a step + bf16 rounding
    for r in (0, 50, 199):                                                        # at most 2^N - 1 levels per group
        assert len(np.unique(y[r, 1])) <= 2 * qmax + 1
    assert np.allclose(np.abs(y).max(-1), amax[..., 0], rtol=2.0 ** -7)           # the largest element survives
    sign_ok = (np.sign(y) == np.sign(xb)) | (y == 0)
    assert sign_ok.all()
    rel = np.sqrt(((y - xb) ** 2).sum() / (xb ** 2).sum())
    assert (rel < 0.012) if n_bits == 8 else (0.03 < rel < 0.2)                   # N(0,1) rows: ~0.7 % / ~11 %


def test_storage_roundtrip_small_case_by_hand(oracle):
    """d = 4, int4 (codes -7..7): row (7, -3.5, 1, 0.49) has scale 1: codes 7, -4 (tie to even), 1, 0."""
    x = np.array([[7.0, -3.5, 1.0, 0.49]], np.float32)
    y = oracle.bf16_bits_to_f32(oracle.storage_roundtrip(oracle.f32_to_bf16_bits(x), 4))
    assert np.array_equal(y, np.array([[7.0, -4.0, 1.0, 0.0]], np.float32))
    x = np.array([[127.0, 63.5, -0.5, 2.4]], np.float32)                          # int8, scale 1: 127, 64, -0, 2
    y = oracle.bf16_bits_to_f32(oracle.storage_roundtrip(oracle.f32_to_bf16_bits(x), 8))
    assert np.array_equal(y, np.array([[127.0, 64.0, -0.0, 2.0]], np.float32))


# ---------------------------------------------------------------------------------------------------------
# Sink + sliding-window leg (Sec. 6, the streaming baseline's mask: n_sink first keys + the last `window`
# keys, positions preserved): the row at absolute position p sees j < n_sink and p - window < j <= p.
# ---------------------------------------------------------------------------------------------------------
def _brute_window(Q, K, V, scale, n_sink, window):
    """Pure python loops over the visible set, nothing vectorised."""
    T, Hq, d = Q.shape
    G = Hq // K.shape[1]
    out = np.zeros((T, Hq, d))
    for p in range(T):
        seen = [j for j in range(p + 1) if j < n_sink or j > p - window]
        for h in range(Hq):
            g = h // G
            s = [scale * sum(Q[p, h, x] * K[j, g, x] for x in range(d)) for j in seen]
            m = max(s)
            e = [math.exp(v - m) for v in s]
            l = sum(e)
            for a, j in enumerate(seen):
                for x in range(d):
                    out[p, h, x] += e[a] / l * V[j, g, x]
    return out


def _window_mask(T, n_sink, window):
    i = np.arange(T)[:, None]
    j = np.arange(T)[None, :]
    return (j <= i) & ((j < n_sink) | (j > i - window))


@pytest.mark.parametrize("n_sink,window", [(0, 1), (0, 4), (2, 3), (4, 5), (1, 30), (3, 1)])
def test_window_brute_force_tiny(oracle, n_sink, window):
    T, Hq, Hkv, d = 14, 4, 2, 8
    Q, K, V = _rand(T, Hq, Hkv, d, 21)
    ref = _brute_window(Q, K, V, 1 / math.sqrt(d), n_sink, window)
    for chunks in ([T], [1] * T, [5, 9], [3, 3, 3, 5]):
        out, _ = oracle.fold(Q, K, V, chunks, n_sink=n_sink, window=window)
        assert np.abs(out - ref).max() < 1e-13, (chunks, n_sink, window)


@pytest.mark.parametrize("T,Hq,Hkv,d,n_sink,window", [(200, 4, 2, 16, 4, 20), (257, 8, 2, 32, 0, 64), (130, 6, 3, 8, 7, 1),
                                                      (96, 4, 1, 64, 4, 1020)])
def test_window_matches_torch_sdpa_with_explicit_mask(oracle, T, Hq, Hkv, d, n_sink, window):
    Q, K, V = _rand(T, Hq, Hkv, d, 22)
    G = Hq // Hkv
    mask = torch.from_numpy(_window_mask(T, n_sink, window))
    q = torch.from_numpy(Q).permute(1, 0, 2)[None]
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(G, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v, attn_mask=mask)[0].permute(1, 0, 2).numpy()
    for chunks in ([T], [64] * (T // 64) + ([T % 64] if T % 64 else []), [T - 1, 1]):
        out, lse = oracle.fold(Q, K, V, chunks, n_sink=n_sink, window=window)
        assert np.abs(out - ref).max() < 1e-12
    # log-sum-exp over exactly the visible keys
    S = np.einsum("ihx,jhx->hij", Q, np.repeat(K, G, axis=1)) / math.sqrt(d)
    S = np.where(_window_mask(T, n_sink, window)[None], S, -np.inf)
    want = np.log(np.exp(S - S.max(-1, keepdims=True)).sum(-1)) + S.max(-1)
    assert np.abs(lse - want.T).max() < 1e-12


def test_window_that_covers_everything_is_the_plain_step(oracle):
    """window >= length: no key is hidden, and the result is the plain step's bit for bit."""
    T, Hq, Hkv, d = 150, 4, 2, 16
    Q, K, V = _rand(T, Hq, Hkv, d, 23)
    plain, plain_lse = oracle.fold(Q, K, V, [50, 50, 50])
    for n_sink, window in ((0, T), (0, 10 * T), (5, T), (T, 1), (T + 7, 3)):      # sinks alone can cover everything too
        out, lse = oracle.fold(Q, K, V, [50, 50, 50], n_sink=n_sink, window=window)
        assert np.array_equal(out, plain) and np.array_equal(lse, plain_lse), (n_sink, window)


def test_window_weights_live_on_the_visible_set_only(oracle):
    T, Hq, Hkv, d, n_sink, window = 90, 4, 2, 8, 3, 11
    Q, K, V = _rand(T, Hq, Hkv, d, 24)
    oc = oracle.OracleCache(Hq, Hkv, d, T)
    oc.step(Q[:40], K[:40], V[:40], 0)
    out, lse, w = oc.step(Q[40:], K[40:], V[40:], 40, want_weights=True, n_sink=n_sink, window=window)
    mask = _window_mask(T, n_sink, window)[40:]                                   # [50][T]
    assert np.all(w[:, :, :][~np.broadcast_to(mask[:, None, :], w.shape)] == 0.0)  # exactly zero outside
    assert np.all(w[np.broadcast_to(mask[:, None, :], w.shape)] > 0.0)
    assert np.abs(w.sum(-1) - 1).max() < 1e-14
    assert (mask.sum(-1) == n_sink + window).all()                                # 3 sinks + 11 recent keys per row
    G = Hq // Hkv
    assert np.abs(np.einsum("rhj,jhx->rhx", w, np.repeat(V, G, axis=1)) - out).max() < 1e-13


def test_window_closed_forms(oracle):
    T, Hq, Hkv, d = 120, 4, 2, 8
    Q, K, V = _rand(T, Hq, Hkv, d, 25)
    # window 1, no sinks: every row sees its own key only
    out, lse = oracle.fold(Q, K, V, [40, 80], n_sink=0, window=1)
    G = Hq // Hkv
    assert np.array_equal(out, np.repeat(V, G, axis=1))
    s_own = np.einsum("ihx,ihx->ih", Q, np.repeat(K, G, axis=1)) / math.sqrt(d)
    assert np.abs(lse - s_own).max() < 1e-13
    # all keys equal: uniform weights over the visible set -> mean of the visible V rows
    Kc = np.broadcast_to(K[:1], K.shape).copy()
    n_sink, window = 2, 9
    out, lse = oracle.fold(Q, Kc, V, [30, 30, 60], n_sink=n_sink, window=window)
    mask = _window_mask(T, n_sink, window)
    want = (mask[:, :, None, None] * V[None]).sum(1) / mask.sum(1)[:, None, None]  # [T][Hkv][d]
    assert np.abs(out - np.repeat(want, G, axis=1)).max() < 1e-13


def test_window_pins_discriminate_planted_mistakes(oracle):
    """Plausible mistakes in the visibility rule move the result by far more than the pins' tolerances."""
    T, Hq, Hkv, d, n_sink, window = 80, 4, 2, 8, 4, 10
    Q, K, V = _rand(T, Hq, Hkv, d, 26)
    good, _ = oracle.fold(Q, K, V, [T], n_sink=n_sink, window=window)
    wrong_rules = {
        "window one key too long": lambda i, j: (j <= i) & ((j < n_sink) | (j >= i - window)),
        "window one key too short": lambda i, j: (j <= i) & ((j < n_sink) | (j > i - window + 1)),
        "sinks forgotten": lambda i, j: (j <= i) & (j > i - window),
        "one sink too many": lambda i, j: (j <= i) & ((j <= n_sink) | (j > i - window)),
        "window counted from the chunk end, not the row": lambda i, j: (j <= i) & ((j < n_sink) | (j > T - 1 - window)),
    }
    G = Hq // Hkv
    i = np.arange(T)[:, None]
    j = np.arange(T)[None, :]
    for name, rule in wrong_rules.items():
        mask = rule(i, j)
        S = np.einsum("ihx,jhx->hij", Q, np.repeat(K, G, axis=1)) / math.sqrt(d)
        S = np.where(mask[None], S, -np.inf)
        P = np.exp(S - S.max(-1, keepdims=True))
        P /= P.sum(-1, keepdims=True)
        bad = np.einsum("hij,jhx->ihx", P, np.repeat(V, G, axis=1))
        assert np.abs(bad - good).max() > 1e-3, name
