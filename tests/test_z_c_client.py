"""The library driven by a plain-C program (no Python, no PyTorch, hipMalloc'd buffers, caller-owned K/V storage,
default stream): what it fed in and what it got back, read from its files, against the oracle."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from paper_2605_12471_amd import build as B

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Hq,Hkv,d,bf16,chunks", [
    (8, 2, 128, 1, [96, 96, 50, 1]),
    (4, 1, 64, 0, [128, 7, 64]),
    (32, 8, 128, 1, [512, 300]),
])
def test_c_client_fold_against_the_oracle(oracle, tmp_path, Hq, Hkv, d, bf16, chunks):
    if not os.path.exists(B.C_CLIENT_PATH):
        pytest.skip("the C client is not built (python __graft_entry__.py builds it next to the library)")
    exe = B.C_CLIENT_PATH
    env = dict(os.environ, LD_LIBRARY_PATH=B.LIB_DIR + os.pathsep + os.environ.get("LD_LIBRARY_PATH", ""))
    if not os.access(exe, os.X_OK):                      # a copy of the tree that dropped the mode bits
        exe = str(tmp_path / "kvfold_c_client")
        shutil.copyfile(B.C_CLIENT_PATH, exe)
        os.chmod(exe, 0o755)
    run = subprocess.run([exe, str(tmp_path), str(Hq), str(Hkv), str(d), str(bf16), "20260512",
                          *map(str, chunks)], capture_output=True, text=True, timeout=100, env=env)
    assert run.returncode == 0, run.stdout + run.stderr
    assert run.stdout.strip().endswith("ok")
    T = sum(chunks)
    et = np.uint16 if bf16 else np.float32

    def load(name, heads):
        return np.fromfile(tmp_path / name, dtype=et).reshape(T, heads, d)

    def wide(x):
        return (oracle.bf16_bits_to_f32(x) if bf16 else x).astype(np.float64)

    q, k, v, out = load("q.bin", Hq), load("k.bin", Hkv), load("v.bin", Hkv), load("out.bin", Hq)
    lse = np.fromfile(tmp_path / "lse.bin", dtype=np.float32)
    assert np.abs(wide(q)).max() <= 2.0 and np.unique(wide(k)).size > 30          # the inputs are what the client says
    oc = oracle.OracleCache(Hq, Hkv, d, T, store_dtype=et)
    pos = lse_pos = 0
    for C in chunks:
        ref, ref_lse = oc.step(wide(q[pos:pos + C]), k[pos:pos + C], v[pos:pos + C], pos)
        err = np.abs(wide(out[pos:pos + C]) - ref).max()
        assert err <= (2e-2 if bf16 else 1e-5), f"chunk at {pos}: max|out-oracle| = {err}"
        got_lse = lse[lse_pos:lse_pos + Hq * C].reshape(Hq, C).T
        assert np.abs(got_lse - ref_lse).max() <= (2e-2 if bf16 else 1e-5)
        pos += C
        lse_pos += Hq * C
    ck = np.fromfile(tmp_path / "cache_k.bin", dtype=et).reshape(Hkv, T, d)
    cv = np.fromfile(tmp_path / "cache_v.bin", dtype=et).reshape(Hkv, T, d)
    assert np.array_equal(ck, oc.k_bits[:, :T]) and np.array_equal(cv, oc.v_bits[:, :T])
