"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the header
declares, validates configurations and plans chunks, and refuses bad arguments with error codes."""
import ctypes
import os
import re

import pytest

import paper_2409_11155_amd as iso

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _good_cfg(**over):
    kw = dict(hidden=256, n_q_heads=4, n_kv_heads=4, head_dim=64, ffn=688, dtype=iso.ISO_F32, max_seq=128)
    kw.update(over)
    return iso.make_cfg(**kw)


def test_library_exports_every_declared_symbol():
    lib = iso.load()
    with open(os.path.join(ROOT, "include", "iso.h")) as f:
        header = f.read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(iso_[a-z0-9_]+)\s*\(", header))
    assert declared, "no declarations parsed"
    assert declared == set(iso.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_validate_cfg_accepts_the_workloads_and_rejects_bad_fields():
    import iso_inputs
    for wl in iso_inputs.WORKLOADS.values():
        cfg = iso.make_cfg(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.dtype, wl.seq)
        assert iso.validate_cfg(cfg) == iso.ISO_OK, wl.name
    assert iso.validate_cfg(_good_cfg(hidden=250)) == iso.ISO_ERR_SHAPE
    assert iso.validate_cfg(_good_cfg(ffn=0)) == iso.ISO_ERR_SHAPE
    assert iso.validate_cfg(_good_cfg(head_dim=96)) == iso.ISO_ERR_SHAPE
    assert iso.validate_cfg(_good_cfg(n_q_heads=6, n_kv_heads=4)) == iso.ISO_ERR_SHAPE
    assert iso.validate_cfg(_good_cfg(n_kv_heads=0)) == iso.ISO_ERR_SHAPE
    assert iso.validate_cfg(_good_cfg(max_seq=0)) == iso.ISO_ERR_SHAPE
    assert iso.validate_cfg(_good_cfg(dtype=7)) == iso.ISO_ERR_DTYPE
    assert iso.validate_cfg(_good_cfg(rope_base=1.0)) == iso.ISO_ERR_SHAPE
    assert iso.load().iso_validate_cfg(None) == iso.ISO_ERR_NULL
    assert "NULL" in iso.last_error()


def test_plan_chunks():
    cfg = _good_cfg(max_seq=8192, hidden=8192, dtype=iso.ISO_BF16, head_dim=128, n_q_heads=16, n_kv_heads=2, ffn=7168)
    p = iso.plan_chunks(cfg, 8192, 4928)
    assert p.n_chunks == 2
    assert list(p.q_offset) == [0, 4928] and list(p.n_tokens) == [4928, 3264] and list(p.kv_len) == [4928, 8192]
    assert list(p.comm_bytes) == [4928 * 8192 * 2, 3264 * 8192 * 2]
    assert p.workspace_bytes >= 8192 * (2 * 8192 + 2560 + 2048 + 3 * 7168) * 2
    for s in (0, 8192):
        p = iso.plan_chunks(cfg, 8192, s)
        assert p.n_chunks == 1 and p.n_tokens[0] == 8192 and p.kv_len[0] == 8192
    p = iso.plan_chunks(cfg, 100, 1)
    assert list(p.n_tokens) == [1, 99]
    for T, s, code in ((8193, 10, iso.ISO_ERR_WORKSPACE), (100, -1, iso.ISO_ERR_SPLIT), (100, 101, iso.ISO_ERR_SPLIT),
                       (0, 0, iso.ISO_ERR_SHAPE)):
        with pytest.raises(iso.IsoError) as ei:
            iso.plan_chunks(cfg, T, s)
        assert ei.value.code == code


def test_plan_split_balances_cost_like_the_oracles_definition():
    """The library's closed-form cut points against the oracle's cumulative-cost definition (Section 6): equal
    up to the rounding to multiples of 128 (of 1 for short prompts)."""
    import numpy as np
    from oracle import iso_oracle as orc
    for (hidden, nq, nkv, d, ffn) in ((6656, 13, 13, 128, 4480), (8192, 8, 1, 128, 3584), (256, 4, 4, 64, 688)):
        cfg = _good_cfg(max_seq=131072, hidden=hidden, dtype=iso.ISO_BF16, head_dim=d, n_q_heads=nq, n_kv_heads=nkv,
                        ffn=ffn)
        sh = orc.LayerShape(hidden, nq, nkv, d, ffn, 1e-6, 1e4)
        for T, n, r in ((2048, 2, 3.0), (8192, 4, 3.0), (16384, 8, 1.0), (131072, 4, 5.0), (300, 4, 3.0), (37, 8, 2.0)):
            got = iso.plan_split(cfg, T, n, r)
            want = orc.balanced_cuts(sh, T, n, r)
            align = 128 if T >= 256 * n else 1
            assert len(got) == n - 1 and all(b > a for a, b in zip([0] + got, got + [T]))
            assert all(g % align == 0 for g in got)
            assert np.all(np.abs(np.array(got) - want) <= align / 2 + 1), (T, n, got, want)
        assert iso.plan_split(cfg, 4096, 4, 0.0) == iso.plan_split(cfg, 4096, 4, 3.0)      # the default ratio
        assert iso.plan_split(cfg, 4096, 1) == []
        assert iso.plan_split(cfg, 5, 5) == [1, 2, 3, 4]
    for T, n, code in ((0, 2, iso.ISO_ERR_SHAPE), (100, 0, iso.ISO_ERR_SHAPE), (100, 9, iso.ISO_ERR_SHAPE),
                       (3, 4, iso.ISO_ERR_SHAPE), (131073, 2, iso.ISO_ERR_WORKSPACE)):
        with pytest.raises(iso.IsoError) as ei:
            iso.plan_split(cfg, T, n)
        assert ei.value.code == code


def test_bench_refuses_more_than_one_gpu():
    import subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)


def test_plan_chunk_count():
    cfg = _good_cfg(max_seq=131072, hidden=8192, dtype=iso.ISO_BF16, head_dim=128, n_q_heads=8, n_kv_heads=1, ffn=3584)
    assert [iso.plan_chunk_count(cfg, T) for T in (1, 511, 512, 2048, 4096, 8192, 16384, 32768, 131072)] == \
        [1, 1, 2, 2, 2, 4, 8, 8, 8]
    for T in (512, 3000, 20000, 131072):        # the count always fits the planner and the prompt
        n = iso.plan_chunk_count(cfg, T)
        assert 1 <= n <= iso.ISO_MAX_CHUNKS and len(iso.plan_split(cfg, T, n)) == n - 1
    for T, code in ((0, iso.ISO_ERR_SHAPE), (131073, iso.ISO_ERR_WORKSPACE)):
        with pytest.raises(iso.IsoError) as ei:
            iso.plan_chunk_count(cfg, T)
        assert ei.value.code == code


def test_gemm_launch_plan_choices_and_invariants():
    """Host logic that picks the projection kernel: stream-K only with enough k depth per team and only where whole
    tiles would fill their rounds of the chip to less than 85 %, its grid a whole number of teams per XCD and never
    larger than the device, the team size a divisor of the tile rows."""
    SK, T256, T128 = iso.ISO_GEMM_STREAMK, iso.ISO_GEMM_TILE_256, iso.ISO_GEMM_TILE_128
    # the projections of the 30B TP=4 chunk (M = 1024) and of the 70B TP=4 chunk (M = 4096) on 256 compute units
    assert iso.gemm_launch_plan(1024, 8960, 6656) == (SK, 4, 256)          # gate/up: 35 columns x 104 slices / 64 teams
    assert iso.gemm_launch_plan(1024, 6656, 1664)[0] == T128               # o_proj: only 10 slices per team
    assert iso.gemm_launch_plan(1024, 6656, 4480) == (SK, 4, 256)          # down: 28 slices per team
    assert iso.gemm_launch_plan(2048, 8192, 1024)[0] == T256               # 70B TP=8 o_proj: 16 slices per team
    assert iso.gemm_launch_plan(4096, 8192, 7168) == (T256, 1, 512)       # 512 whole tiles: two full rounds, no stream-K
    assert iso.gemm_launch_plan(4096, 14336, 8192) == (T256, 1, 896)      # 3.5 rounds of whole tiles fill 87.5 % of four
    assert iso.gemm_launch_plan(4096, 2560, 8192) == (SK, 8, 256)         # 160 tiles: 62 % of one round
    assert iso.gemm_launch_plan(3072, 8192, 4096) == (SK, 4, 256)         # 384 tiles: 75 % of two rounds
    assert iso.gemm_launch_plan(4096, 8192, 7168, num_cu=0) == (T256, 1, 512)   # no workspace: one tile per workgroup
    assert iso.gemm_launch_plan(300, 257 * 8, 1000)[0] in (iso.ISO_GEMM_STAGED, iso.ISO_GEMM_SIMPLE)   # K % 64 != 0
    assert iso.gemm_launch_plan(7, 12, 9)[0] == iso.ISO_GEMM_SIMPLE
    import random
    rnd = random.Random(3)
    for _ in range(3000):
        M, N, K = rnd.randint(1, 9000), 8 * rnd.randint(1, 2000), 64 * rnd.randint(1, 130)
        cus = rnd.choice([8, 64, 104, 256, 304])
        kind, team, grid = iso.gemm_launch_plan(M, N, K, cus)
        tiles_m, tiles_n, nk = -(-M // 256), -(-N // 256), K // 64
        if kind == SK:
            assert team in (1, 2, 4, 8) and tiles_m % team == 0
            assert 0 < grid <= cus and grid % (8 * team) == 0
            teams = grid // team
            assert (tiles_m // team) * tiles_n * nk // teams >= 20
            rounds = -(-tiles_m * tiles_n // cus)
            assert tiles_m * tiles_n * 100 < 85 * rounds * cus       # whole tiles would leave the chip idle
        elif kind == T256:
            assert grid == tiles_m * tiles_n and grid >= 128
        else:
            assert kind == T128 and grid == (-(-M // 128)) * (-(-N // 128))
    for args, code in (((0, 8, 64, 256), iso.ISO_ERR_SHAPE), ((8, 8, 64, -1), iso.ISO_ERR_SHAPE)):
        with pytest.raises(iso.IsoError) as ei:
            iso.gemm_launch_plan(*args)
        assert ei.value.code == code


def test_null_context_and_null_out_are_refused_without_touching_a_device():
    lib = iso.load()
    w = iso.IsoWeights()
    assert lib.iso_layer_prefill(None, ctypes.byref(w), None, None, None, 4, 2, 0, 0) == iso.ISO_ERR_NULL
    assert lib.iso_stack_prefill(None, ctypes.byref(w), 1, None, None, None, 4, 2, 0, 0) == iso.ISO_ERR_NULL
    assert lib.iso_attn_chunk(None, None, None, None, None, 1, 0, 1, None) == iso.ISO_ERR_NULL
    assert lib.iso_gemm_rowpar(None, None, None, None, 1, 1, 8, None, None) == iso.ISO_ERR_NULL
    assert lib.iso_rmsnorm(None, None, None, None, 1, None) == iso.ISO_ERR_NULL
    assert lib.iso_residual_rmsnorm(None, None, None, None, None, 1, None) == iso.ISO_ERR_NULL
    assert lib.iso_rope_kv_write(None, None, None, None, 1, 0, None) == iso.ISO_ERR_NULL
    assert lib.iso_swiglu(None, None, None, 1, None) == iso.ISO_ERR_NULL
    assert lib.iso_sync(None) == iso.ISO_ERR_NULL
    assert lib.iso_destroy(None) == iso.ISO_ERR_NULL
    assert lib.iso_set_flags(None, 0) == iso.ISO_ERR_NULL
    assert lib.iso_host_sink(None) is None
    cfg = _good_cfg()
    assert lib.iso_create(None, ctypes.byref(cfg), None, None) == iso.ISO_ERR_NULL
    handle = ctypes.c_void_p(1234)
    bad = _good_cfg(head_dim=80)
    assert lib.iso_create(ctypes.byref(handle), ctypes.byref(bad), None, None) == iso.ISO_ERR_SHAPE
    assert handle.value is None          # *out is cleared on failure


@pytest.mark.skipif(iso.device_count() > 0, reason="checks the no-device error path")
def test_create_without_a_device_reports_a_hip_error():
    with pytest.raises(iso.IsoError) as ei:
        iso.Context(_good_cfg())
    assert ei.value.code == iso.ISO_ERR_HIP


@pytest.mark.skipif(iso.device_count() > 0, reason="checks the no-device error path")
def test_plumbing_without_a_device_reports_errors_not_crashes():
    lib = iso.load()
    assert iso.device_count() == 0
    p = ctypes.c_void_p(77)
    assert lib.iso_dev_alloc(ctypes.byref(p), 16) == iso.ISO_ERR_HIP and p.value is None
    assert lib.iso_dev_alloc(None, 16) == iso.ISO_ERR_NULL
    assert lib.iso_stream_create(None) == iso.ISO_ERR_NULL
    assert lib.iso_copy_h2d(None, None, 4) == iso.ISO_ERR_NULL
    assert lib.iso_dev_free(None) == iso.ISO_OK and lib.iso_host_free(None) == iso.ISO_OK
