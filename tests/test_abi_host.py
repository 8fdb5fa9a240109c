"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and
every error path that can be decided without a GPU returns the documented status."""
import ctypes
import os
import re

import pytest

import paper_2605_12471_amd as kv
from paper_2605_12471_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(kv.lib_path()):
        build.build_library()
    return kv.load_library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "kvfold.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvfold_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"kvfold_cache_create", "kvfold_step", "kvfold_step_ex", "kvfold_cache_destroy"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in kvfold.h but not exported"


def test_python_binding_has_the_same_names():
    for n in _declared_functions():
        assert hasattr(kv, n), f"binding lacks {n}"


def test_struct_layout_matches_header():
    # field order and natural alignment of kvfold_config_t (64-bit ABI)
    c = binding.kvfold_config_t
    assert ctypes.sizeof(c) == 64
    assert c.capacity_tokens.offset == 24 and c.kv_buffer.offset == 48 and c.kv_buffer_bytes.offset == 56


def test_bytes_required_matches_paper_accounting(lib):
    """Tab. 4 caption: 32 layers x 8 KV heads x 128 dims x (K,V) x 2 bytes = 131,072 bytes per token."""
    vals = {}
    rows = []
    for line in open(os.path.join(ROOT, "tests", "golden", "paper_cache_accounting.txt")):
        if line.startswith("#") or not line.strip():
            continue
        parts = line.split()
        if parts[0] == "kv_gb":
            rows.append((int(parts[1]), float(parts[2])))
        elif len(parts) == 2:
            vals[parts[0]] = int(parts[1])
    cfg = binding.make_config(vals["layers"], 32, vals["kv_heads"], vals["head_dim"], 1, 1, kv.KVFOLD_BF16)
    assert kv.kvfold_cache_bytes_required(cfg) == vals["bytes_per_token"]
    for tokens, gb in rows:
        cfg.capacity_tokens = tokens
        need = kv.kvfold_cache_bytes_required(cfg)
        assert need == tokens * vals["bytes_per_token"]
        assert abs(need / 1e9 - gb) < 0.006          # the table prints two decimals
    # the streaming baseline's configuration (Sec. 6): 4 sinks + 1020 recent tokens fill its 1024-token cache
    assert vals["stream_sinks"] + vals["stream_window"] == vals["stream_capacity"] == 1024
    cfg.capacity_tokens = 131072
    assert kv.kvfold_cache_bytes_required(cfg) == 17179869184   # 16 GiB exactly
    # fp32 doubles it
    cfg.dtype = kv.KVFOLD_F32
    assert kv.kvfold_cache_bytes_required(cfg) == 2 * 17179869184


@pytest.mark.parametrize("mutate,status", [
    (lambda c: setattr(c, "struct_size", 8), -1),
    (lambda c: setattr(c, "n_layers", 0), -1),
    (lambda c: setattr(c, "chunk_tokens", 0), -1),
    (lambda c: setattr(c, "capacity_tokens", 0), -1),
    (lambda c: setattr(c, "device", -1), -1),
    (lambda c: setattr(c, "softmax_scale", -1.0), -1),
    (lambda c: setattr(c, "softmax_scale", float("nan")), -1),
    (lambda c: setattr(c, "chunk_tokens", 4096), -1),           # chunk larger than capacity
    (lambda c: setattr(c, "kv_buffer", 0x1001), -1),            # misaligned caller buffer
    (lambda c: setattr(c, "head_dim", 96), -5),
    (lambda c: setattr(c, "n_q_heads", 7), -5),                 # not a multiple of Hkv
    (lambda c: setattr(c, "dtype", 7), -5),
    (lambda c: setattr(c, "capacity_tokens", 1 << 31), -5),
])
def test_create_rejects_bad_config_before_touching_the_gpu(lib, mutate, status):
    cfg = binding.make_config(2, 8, 2, 128, 64, 1024, kv.KVFOLD_BF16)
    mutate(cfg)
    rc, h = kv.kvfold_cache_create(cfg)
    assert rc == status and h is None
    assert kv.kvfold_cache_bytes_required(cfg) == 0


def test_caller_buffer_too_small_is_oom(lib):
    cfg = binding.make_config(1, 8, 2, 128, 64, 1024, kv.KVFOLD_BF16, kv_buffer=0x10000, kv_buffer_bytes=1024)
    rc, h = kv.kvfold_cache_create(cfg)
    assert rc == -6 and h is None


def test_null_handles(lib):
    assert lib.kvfold_cache_create(None, None) == -1
    assert kv.kvfold_cache_destroy(None) == 0                     # NULL is a no-op
    assert kv.kvfold_cache_length(None, 0) == -1
    assert kv.kvfold_step(None, 0, 1, 1, 1, 0, 1, 0) == -1
    assert kv.kvfold_step_ex(None, 0, 1, 1, 1, 1, 0, 1, None, 0) == -1
    assert kv.kvfold_step_rope(None, 0, 1, 1, 1, 1, 0, 16, 16, 1, None, 0) == -1
    assert kv.kvfold_step_rope(None, 0, 1, 1, 1, 1, 0, None, None, 1, None, 0) == -1
    assert kv.kvfold_step_window(None, 0, 16, 16, 16, 1, 0, 4, 1020, 16, None, 0) == -1
    assert kv.kvfold_step_window(None, 0, 16, 16, 16, 1, 0, -1, 1020, 16, None, 0) == -1
    assert kv.kvfold_step_window(None, 0, 16, 16, 16, 1, 0, 4, 0, 16, None, 0) == -1
    assert kv.kvfold_step_noalloc(None, 0, 16, 16, 16, 1, 0, 16, None, 0) == -1
    assert kv.kvfold_cache_set_length(None, 0, 0) == -1
    assert kv.kvfold_cache_truncate(None, 0, 0) == -1
    assert kv.kvfold_cache_set_tuning(None, 0, 0) == -1
    assert kv.kvfold_cache_set_storage_roundtrip(None, 8) == -1
    assert kv.kvfold_cache_plan(None, 1, 1)[0] == -1
    assert kv.kvfold_cache_view(None, 0)[0] == -1
    assert kv.kvfold_cache_profile_begin(None, 1) == -1
    assert kv.kvfold_cache_profile_end(None)[0] == -1


def test_launch_plans_of_the_benchmark_configurations(lib):
    """The host-side planner on a 256-CU part (no GPU needed): the geometry each benchmark workload is timed in."""
    def plan(Hq, Hkv, d, C, L, dtype=kv.KVFOLD_BF16, cap=131072):
        cfg = binding.make_config(1, Hq, Hkv, d, C, cap, dtype)
        rc, pl = kv.kvfold_plan_for(cfg, 256, C, L)
        assert rc == 0
        return pl.n_workgroups, pl.n_splits, pl.units_per_wave
    # config 2 (C=2048 to 16K): first step one unit per wavefront, two workgroups per CU; then one round of 256
    assert plan(32, 8, 128, 2048, 2048) == (512, 1, 1)
    for L in (4096, 8192, 16384):
        assert plan(32, 8, 128, 2048, L) == (256, 1, 2)
    # config 3 (C=256 to 128K): the prefix is split until the chip is full: 32 workgroups x 8
    assert plan(32, 8, 128, 256, 131072) == (256, 8, 2)
    # config 4 (C=4096 to 128K): two rounds of 256, unsplit
    assert plan(32, 8, 128, 4096, 131072) == (512, 1, 2)
    # config 5 (G=7, C=2048): 224 busy CUs of 256 beat any split on the power-limited chip
    assert plan(28, 4, 128, 2048, 65536, cap=65536) == (224, 1, 2)
    assert plan(28, 4, 128, 8192, 65536, cap=65536) == (1792, 2, 2)
    # config 5 at C=128: the 28 units of a G=7 head fill 3.5 two-unit workgroups; seven one-unit workgroups and nine
    # pieces on 252 CUs are faster (measured: +9 % on the fold)
    assert plan(28, 4, 128, 128, 65536, cap=65536) == (252, 9, 1)
    # decode-shaped steps against 128K: one unit per wavefront, 512 workgroups (two per CU)
    w, s, u = plan(32, 8, 128, 16, 131072)
    assert (w, s, u) == (512, 64, 1)
    w, s, u = plan(32, 8, 128, 1, 131072)
    assert u == 1 and 63 <= s <= 64 and w == 8 * s
    # fp32 mode: one unit per wavefront always
    assert plan(4, 1, 64, 128, 512, kv.KVFOLD_F32, cap=512)[2] == 1
    # argument errors
    cfg = binding.make_config(1, 32, 8, 128, 256, 1024, kv.KVFOLD_BF16)
    assert kv.kvfold_plan_for(cfg, 256, 257, 1024)[0] == -1      # more rows than the chunk size
    assert kv.kvfold_plan_for(cfg, 256, 256, 2048)[0] == -1      # beyond the capacity
    assert kv.kvfold_plan_for(cfg, 0, 256, 1024)[0] == -1
    assert kv.kvfold_plan_for(None, 256, 256, 1024)[0] == -1
    assert kv.kvfold_plan_for(cfg, 256, 256, 1024, n_sink=-1, window=8)[0] == -1
    assert kv.kvfold_plan_for(cfg, 256, 256, 1024, n_sink=0, window=-1)[0] == -1
    assert load_raw_plan_for_null_out(cfg) == -1


def load_raw_plan_for_null_out(cfg):
    return kv.load_library().kvfold_plan_for(ctypes.byref(cfg), 256, 256, 1024, 0, 0, None)


def test_fused_append_decision_at_its_limits(lib):
    """The attention kernel appends by itself only when it can address the chunk's rows, [C][Hkv][d], with 32-bit
    byte offsets (C * Hkv * d * 2 bytes below 2^32) and the cache is bf16; everything else goes through the
    separate append kernel.  Pinned through the host-only planner."""
    def fused(Hq, Hkv, d, C, L, dtype=kv.KVFOLD_BF16):
        cfg = binding.make_config(1, Hq, Hkv, d, C, max(L, C), dtype)
        rc, pl = kv.kvfold_plan_for(cfg, 256, C, L)
        assert rc == 0
        return pl.fused_append
    assert fused(32, 8, 128, 2048, 16384) == 1
    assert fused(32, 8, 128, 2048, 2048 + 63) == 1              # any cache length: a straddling tile is filled from both sides
    assert fused(32, 8, 128, 1, 131072) == 1                    # decode-shaped steps: two launches (attention, merge)
    assert fused(4, 1, 64, 128, 512, kv.KVFOLD_F32) == 0
    # Hkv = 8, d = 128: a chunk row is 2048 bytes, 2^32 bytes are 2,097,152 tokens
    assert fused(8, 8, 128, 2097151, 2097151) == 1
    assert fused(8, 8, 128, 2097152, 2097152) == 0
    assert fused(8, 8, 128, 4000000, 4000000) == 0
    # Hkv = 64, d = 128: 16 KiB per token, the limit is 262,144 tokens; d = 64: 524,288
    assert fused(64, 64, 128, 262143, 262143) == 1
    assert fused(64, 64, 128, 262144, 262144) == 0
    assert fused(64, 64, 64, 524287, 524287) == 1
    assert fused(64, 64, 64, 524288, 524288) == 0
    # a ragged last chunk of a config whose full chunk is too large is fused again
    cfg = binding.make_config(1, 8, 8, 128, 4000000, 8000000, kv.KVFOLD_BF16)
    assert kv.kvfold_plan_for(cfg, 256, 4000000, 4000000)[1].fused_append == 0
    assert kv.kvfold_plan_for(cfg, 256, 1000000, 5000000 - 5000000 % 64 + 1000000 - 1000000 % 64)[1].fused_append == 1


def test_create_rejects_more_kv_heads_than_the_append_grid_holds(lib):
    cfg = binding.make_config(1, 32768, 32768, 64, 1, 64, kv.KVFOLD_BF16)
    assert kv.kvfold_cache_create(cfg)[0] == -5
    cfg = binding.make_config(1, 32767, 32767, 64, 1, 64, kv.KVFOLD_BF16)
    assert kv.kvfold_cache_bytes_required(cfg) > 0


def test_window_plans_do_work_proportional_to_the_window(lib):
    """Sink + sliding-window step (4 sinks + 1020 recent tokens, Sec. 6) against a 128K cache: the tiles a
    workgroup walks cover the sink tile, the window and its own rows, not the cache."""
    cfg = binding.make_config(1, 32, 8, 128, 256, 131072, kv.KVFOLD_BF16)
    rc, pl = kv.kvfold_plan_for(cfg, 256, 256, 131072, n_sink=4, window=1020)
    assert rc == 0
    tiles = pl.n_splits * pl.tiles_per_split
    assert 17 <= tiles <= 20 * pl.n_splits and pl.tiles_per_split <= 20      # 1 sink tile + (1020 + 64 rows) / 64 + edges
    assert pl.pair_units == 0 and pl.pair_order == 0
    rc, plain = kv.kvfold_plan_for(cfg, 256, 256, 131072)
    assert plain.n_splits * plain.tiles_per_split >= 2048
    # a window wider than the cache: the plain key range
    rc, wide = kv.kvfold_plan_for(cfg, 256, 256, 131072, n_sink=0, window=1 << 20)
    assert wide.n_splits * wide.tiles_per_split >= 2048


def test_status_strings(lib):
    seen = {kv.kvfold_status_string(s) for s in range(0, -9, -1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert kv.kvfold_status_string(-99) == "unknown status"


def test_kernels_use_no_scratch_memory():
    """Register-resident kernels: the compiler's resource report must show no scratch and no spills."""
    if not os.path.exists(build.RESOURCE_REPORT):
        build.build_library()
    text = open(build.RESOURCE_REPORT).read()
    blocks = text.split("Function Name: ")[1:]
    names = [b.splitlines()[0] for b in blocks]
    assert any("attn_bf16_kernel" in n for n in names) and any("attn_f32_kernel" in n for n in names)
    for b in blocks:
        name = b.splitlines()[0]
        scratch = int(re.search(r"ScratchSize \[bytes/lane\]: (\d+)", b).group(1))
        spill = int(re.search(r"VGPRs Spill: (\d+)", b).group(1))
        assert scratch == 0 and spill == 0, f"{name}: scratch {scratch} B/lane, {spill} spilled VGPRs"
        if "attn_bf16_kernelILi128ELi2" in name:   # the flagship kernel: one wave per SIMD, O (128) and Q (64) in AGPRs
            assert int(re.search(r"AGPRs: (\d+)", b).group(1)) >= 192


def test_header_is_plain_c_and_the_c_client_builds(tmp_path):
    """include/kvfold.h compiles as strict C99 on its own (no C++ or HIP in the interface), and the plain-C caller of the
    library compiles with gcc and links against the built library."""
    import subprocess
    from paper_2605_12471_amd import build as B
    src = tmp_path / "only_header.c"
    src.write_text('#include "kvfold.h"\nint main(void) { kvfold_config_t c; c.struct_size = sizeof c; return (int)c.struct_size * 0; }\n')
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I" + B.INCLUDE_DIR, "-c", str(src),
                    "-o", str(tmp_path / "only_header.o")], check=True)
    assert os.path.exists(B.build_c_client())
