"""GPU parity: every entry point of libiso against the CPU oracle on the same seeded inputs.

Tolerances (metric: max |got - ref| / max(|ref|, rms(ref)), see oracle.max_rel_err):
  fp32 path  : 1e-4 for the whole layer; single steps 2e-5 (fp32 accumulation over <= 1e3 terms).
  bf16 path  : 2e-2 for the whole layer.  Single steps: the output rounding alone is 2^-8 = 3.9e-3
               relative; steps that also round an intermediate (attention probabilities, SwiGLU input)
               get 1e-2.
"""
import numpy as np
import pytest
import torch

import iso_inputs
import paper_2409_11155_amd as iso
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

TOL_LAYER = {"f32": 1e-4, "bf16": 2e-2}
TOL_STEP = {"f32": 2e-5, "bf16": 1e-2}
DEV = "cuda:0"


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu", torch.float64).numpy()


def shape_of(hidden, nq, nkv, d, ffn, eps=1e-6, base=10000.0):
    return orc.LayerShape(hidden, nq, nkv, d, ffn, eps, base)


def make_ctx(hidden, nq, nkv, d, ffn, dtype, max_seq, two_streams=True):
    cfg = iso.make_cfg(hidden, nq, nkv, d, ffn, dtype, max_seq)
    s0 = torch.cuda.Stream(device=DEV)
    s1 = torch.cuda.Stream(device=DEV) if two_streams else s0
    return iso.Context(cfg, s0, s1)


def dtype_name(dt):
    return "f32" if dt == torch.float32 else "bf16"


# ------------------------------------------------------------------------------ element-wise steps

@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,H", [(1, 256), (37, 1000), (130, 8192), (5, 16384)])
def test_rmsnorm_and_residual_rmsnorm(dt, T, H):
    torch.manual_seed(T * 7 + H)
    x = torch.randn(T, H).to(dt)
    delta = (0.5 * torch.randn(T, H)).to(dt)
    g = (1 + 0.1 * torch.randn(H)).to(dt)
    with make_ctx(H, 4, 4, 64, 64, dt, 256) as ctx:
        xd, dd, gd = x.to(DEV), delta.to(DEV), g.to(DEV)
        y = torch.empty_like(xd)
        ctx.rmsnorm(xd, gd, y, T, ctx.stream0)
        ctx.sync()
        tol = TOL_STEP[dtype_name(dt)]
        assert orc.max_rel_err(f64(y), orc.rmsnorm(f64(x), f64(g), 1e-6)) <= tol
        # fused: x += delta (in place), y = norm(x)
        y2 = torch.empty_like(xd)
        ctx.residual_rmsnorm(xd, dd, gd, y2, T, ctx.stream0)
        ctx.sync()
        x1 = f64(x) + f64(delta)
        assert orc.max_rel_err(f64(xd), x1) <= tol
        assert orc.max_rel_err(f64(y2), orc.rmsnorm(x1, f64(g), 1e-6)) <= tol
        # residual only
        xd2 = x.to(DEV)
        ctx.residual_rmsnorm(xd2, dd, None, None, T, ctx.stream0)
        ctx.sync()
        assert orc.max_rel_err(f64(xd2), x1) <= tol


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("nq,nkv,d", [(4, 4, 64), (8, 1, 128), (13, 13, 128), (6, 2, 64)])
def test_rope_kv_write(dt, nq, nkv, d):
    Tc, q_offset, max_seq = 70, 41, 128
    torch.manual_seed(nq * 100 + d)
    qkv = torch.randn(Tc, (nq + 2 * nkv) * d).to(dt)
    with make_ctx(256, nq, nkv, d, 64, dt, max_seq) as ctx:
        qd = qkv.to(DEV)
        kc = torch.full((max_seq, nkv, d), 7.0, dtype=dt, device=DEV)
        vc = torch.full((max_seq, nkv, d), 7.0, dtype=dt, device=DEV)
        ctx.rope_kv_write(qd, kc, vc, Tc, q_offset, ctx.stream0)
        ctx.sync()
        pos = np.arange(q_offset, q_offset + Tc)
        ref = f64(qkv)
        q_ref = orc.rope(ref[:, : nq * d].reshape(Tc, nq, d), pos, 10000.0)
        k_ref = orc.rope(ref[:, nq * d:(nq + nkv) * d].reshape(Tc, nkv, d), pos, 10000.0)
        v_ref = ref[:, (nq + nkv) * d:].reshape(Tc, nkv, d)
        tol = TOL_STEP[dtype_name(dt)]
        assert orc.max_rel_err(f64(qd)[:, : nq * d].reshape(Tc, nq, d), q_ref) <= tol
        assert orc.max_rel_err(f64(kc)[q_offset:q_offset + Tc], k_ref) <= tol
        np.testing.assert_array_equal(f64(vc)[q_offset:q_offset + Tc], v_ref)       # v is a copy: bit-exact
        # rows outside the chunk are untouched
        assert torch.all(kc[:q_offset] == 7.0) and torch.all(kc[q_offset + Tc:] == 7.0)
        assert torch.all(vc[:q_offset] == 7.0) and torch.all(vc[q_offset + Tc:] == 7.0)


@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("T,F", [(1, 8), (33, 688), (129, 3584)])
def test_swiglu(dt, T, F):
    torch.manual_seed(F)
    gu = (2.0 * torch.randn(T, 2 * F)).to(dt)
    with make_ctx(256, 4, 4, 64, F, dt, 256) as ctx:
        a = torch.empty(T, F, dtype=dt, device=DEV)
        ctx.swiglu(gu.to(DEV), a, T, ctx.stream0)
        ctx.sync()
        assert orc.max_rel_err(f64(a), orc.swiglu(f64(gu))) <= TOL_STEP[dtype_name(dt)]


# ------------------------------------------------------------------------------ projections

GEMM_SHAPES = [(1, 8, 8), (64, 128, 64), (128, 128, 64), (129, 130, 72), (300, 257, 1000), (77, 768, 256),
               (256, 384, 688), (513, 1280, 2048)]


@pytest.mark.parametrize("dt,flags", [(torch.float32, 0), (torch.bfloat16, 0),
                                      (torch.bfloat16, iso.ISO_FLAG_SIMPLE_GEMM)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_rowpar(dt, flags, M, N, K):
    torch.manual_seed(M + N + K)
    a = torch.randn(M, K).to(dt)
    w = (torch.randn(N, K) * K ** -0.5).to(dt)
    with make_ctx(256, 4, 4, 64, 64, dt, 256) as ctx:
        ctx.set_flags(flags)
        c = torch.zeros(M, N, dtype=dt, device=DEV)
        sink = torch.zeros(M, N, dtype=dt).pin_memory()
        ctx.gemm_rowpar(a.to(DEV), w.to(DEV), c, M, N, K, ctx.stream0, sink.data_ptr())
        ctx.sync()
        ref = orc.linear(f64(a), f64(w))
        assert orc.max_rel_err(f64(c), ref) <= TOL_STEP[dtype_name(dt)]
        assert torch.equal(sink, c.cpu())          # the communication stand-in moved exactly the partial


def test_gemm_rejects_bad_shapes():
    with make_ctx(256, 4, 4, 64, 64, torch.bfloat16, 256) as ctx:
        a = torch.zeros(4, 12, dtype=torch.bfloat16, device=DEV)
        for (M, N, K) in ((4, 4, 12), (0, 4, 8), (4, -1, 8)):
            with pytest.raises(iso.IsoError) as ei:
                ctx.gemm_rowpar(a, a, a, M, N, K, ctx.stream0)
            assert ei.value.code == iso.ISO_ERR_SHAPE


# ------------------------------------------------------------------------------ attention

ATTN_CASES = [
    # Tc, q_offset, kv_len, nq, nkv
    (1, 0, 1, 4, 4),
    (64, 0, 64, 4, 4),
    (128, 0, 128, 8, 1),
    (200, 0, 200, 4, 2),
    (130, 77, 207, 8, 1),        # second chunk: rectangular block + ragged causal block
    (257, 300, 557, 2, 2),
    (33, 500, 533, 13, 13),
    (100, 60, 130, 4, 1),        # kv_len cuts the last rows short
]


@pytest.mark.parametrize("dt,d,flags", [(torch.float32, 64, 0), (torch.float32, 128, 0), (torch.bfloat16, 128, 0),
                                        (torch.bfloat16, 128, iso.ISO_FLAG_SIMPLE_ATTN), (torch.bfloat16, 64, 0)])
@pytest.mark.parametrize("Tc,q_offset,kv_len,nq,nkv", ATTN_CASES)
def test_attn_chunk(dt, d, flags, Tc, q_offset, kv_len, nq, nkv):
    q, k, v = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=Tc + q_offset, dtype=dt)
    with make_ctx(256, nq, nkv, d, 64, dt, 1024) as ctx:
        ctx.set_flags(flags)
        out = torch.zeros(Tc, nq * d, dtype=dt, device=DEV)
        ctx.attn_chunk(q.to(DEV), k.to(DEV), v.to(DEV), out, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        ref = orc.attention_chunk(f64(q), f64(k), f64(v), q_offset, kv_len).reshape(Tc, nq * d)
        tol = TOL_STEP[dtype_name(dt)]
        if dt == torch.bfloat16 and d == 128 and flags == 0:
            # the matrix-core kernel rounds the probabilities to bf16 before the second product:
            # |d out| <= 2^-9 * sum_j p_j |v_j| <= 2^-9 max|v|, on top of the 2^-8 output rounding
            rms = float(np.sqrt(np.mean(ref * ref)))
            tol = 2.0 ** -9 * float(v.abs().max()) / rms + 2.0 ** -8 + 1e-4
        err = orc.max_rel_err(f64(out), ref)
        assert err <= tol, (err, tol)


def test_attn_chunk_rejects_bad_arguments():
    with make_ctx(256, 4, 4, 64, 64, torch.float32, 64) as ctx:
        t = torch.zeros(64, 256, device=DEV)
        for args, code in (((0, 0, 1), iso.ISO_ERR_SHAPE), ((4, -1, 4), iso.ISO_ERR_SHAPE), ((4, 0, 0), iso.ISO_ERR_SHAPE),
                           ((4, 0, 65), iso.ISO_ERR_WORKSPACE), ((65, 0, 4), iso.ISO_ERR_WORKSPACE)):
            with pytest.raises(iso.IsoError) as ei:
                ctx.attn_chunk(t, t, t, t, *args, ctx.stream0)
            assert ei.value.code == code


# ------------------------------------------------------------------------------ whole layer

def run_layer(ctx, w_dev, x_cpu, T, split, nkv, d, max_seq, comm=iso.ISO_COMM_NONE, sched=iso.ISO_SCHED_OVERLAP,
              poison=False):
    x = x_cpu.to(DEV).clone()
    fill = float("nan") if poison else 0.0
    kc = torch.full((max_seq, nkv, d), fill, dtype=x.dtype, device=DEV)
    vc = torch.full((max_seq, nkv, d), fill, dtype=x.dtype, device=DEV)
    torch.cuda.synchronize()
    ctx.layer_prefill(w_dev, x, kc, vc, T, split, comm, sched)
    ctx.sync()
    return x, kc, vc


def test_tiny_f32_layer_unsplit_and_every_tested_split():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_unsplit(f64(x), {k: f64(v) for k, v in w.items()}, sh)
    w_dev = {k: v.to(DEV) for k, v in w.items()}
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, torch.float32, wl.seq) as ctx:
        for split in (0, wl.seq, 64, 1, 127, 33, 77, 100):
            for sched in (iso.ISO_SCHED_OVERLAP, iso.ISO_SCHED_SERIAL):
                for comm in (iso.ISO_COMM_NONE, iso.ISO_COMM_D2H):
                    out, kc, vc = run_layer(ctx, w_dev, x, wl.seq, split, wl.n_kv_heads, wl.head_dim, wl.seq, comm,
                                            sched, poison=True)
                    err = orc.max_rel_err(f64(out), ref["x_out"])
                    assert err <= TOL_LAYER["f32"], (split, sched, comm, err)
                    assert orc.max_rel_err(f64(kc), ref["k_cache"]) <= TOL_STEP["f32"]
                    assert orc.max_rel_err(f64(vc), ref["v_cache"]) <= TOL_STEP["f32"]


def test_tiny_f32_layer_matches_the_oracles_iso_path_too():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_iso(f64(x), {k: f64(v) for k, v in w.items()}, sh, wl.split)
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, torch.float32, wl.seq) as ctx:
        out, _, _ = run_layer(ctx, {k: v.to(DEV) for k, v in w.items()}, x, wl.seq, wl.split, wl.n_kv_heads,
                              wl.head_dim, wl.seq)
        assert orc.max_rel_err(f64(out), ref["x_out"]) <= TOL_LAYER["f32"]


@pytest.mark.parametrize("flags", [0, iso.ISO_FLAG_SIMPLE_GEMM | iso.ISO_FLAG_SIMPLE_ATTN])
@pytest.mark.parametrize("hidden,nq,nkv,ffn,T,splits", [
    (512, 4, 1, 768, 300, (0, 130, 299)),       # GQA, ragged everything
    (384, 3, 3, 200, 257, (128, 1)),            # MHA, odd head count
])
def test_small_bf16_layer_all_rows(flags, hidden, nq, nkv, ffn, T, splits):
    d = 128
    dt = torch.bfloat16
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=11, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=11, dtype=dt)
    ref = orc.layer_unsplit(f64(x), {k: f64(v) for k, v in w.items()}, shape_of(hidden, nq, nkv, d, ffn))
    w_dev = {k: v.to(DEV) for k, v in w.items()}
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 320) as ctx:
        ctx.set_flags(flags)
        for split in splits:
            out, kc, vc = run_layer(ctx, w_dev, x, T, split, nkv, d, 320, iso.ISO_COMM_D2H, poison=True)
            err = orc.max_rel_err(f64(out), ref["x_out"])
            assert err <= TOL_LAYER["bf16"], (split, err)
            # cached K went through three bf16 roundings (norm output, projection output, rotation)
            assert orc.max_rel_err(f64(kc)[:T], ref["k_cache"]) <= TOL_LAYER["bf16"]
            assert orc.max_rel_err(f64(vc)[:T], ref["v_cache"]) <= TOL_LAYER["bf16"]


def test_two_layer_stack_equals_two_oracle_layers():
    hidden, nq, nkv, d, ffn, T, split = 256, 2, 1, 128, 256, 200, 90
    dt = torch.bfloat16
    layers = [iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=20 + l, dtype=dt) for l in range(2)]
    x = iso_inputs.make_hidden(T, hidden, seed=5, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    ref = f64(x)
    for w in layers:
        ref = orc.layer_unsplit(ref, {k: f64(v) for k, v in w.items()}, sh)["x_out"]
    with make_ctx(hidden, nq, nkv, d, ffn, dt, T) as ctx:
        for s in (0, split):
            xd = x.to(DEV).clone()
            kcs = torch.zeros(2, T, nkv, d, dtype=dt, device=DEV)
            vcs = torch.zeros(2, T, nkv, d, dtype=dt, device=DEV)
            torch.cuda.synchronize()
            ctx.stack_prefill([{k: v.to(DEV) for k, v in w.items()} for w in layers], xd, kcs, vcs, T, s,
                              iso.ISO_COMM_D2H)
            ctx.sync()
            # two layers compound the per-layer bf16 error: allow twice the per-layer bound
            assert orc.max_rel_err(f64(xd), ref) <= 2 * TOL_LAYER["bf16"]


def test_kv_event_orders_the_chunks_and_runs_are_bit_identical():
    """Chunk 1 must not read the cache before chunk 0 wrote it (Section 3.1).  The cache starts as NaN, so a
    read that overtook the write would surface as NaN; repeated runs must also agree bit for bit."""
    hidden, nq, nkv, d, ffn, T, split = 1024, 8, 1, 128, 1024, 1024, 512
    dt = torch.bfloat16
    w = {k: v.to(DEV) for k, v in iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=3, dtype=dt).items()}
    x = iso_inputs.make_hidden(T, hidden, seed=3, dtype=dt)
    with make_ctx(hidden, nq, nkv, d, ffn, dt, T) as ctx:
        first = None
        for _ in range(10):
            out, _, _ = run_layer(ctx, w, x, T, split, nkv, d, T, iso.ISO_COMM_D2H, poison=True)
            assert not torch.isnan(out).any()
            if first is None:
                first = out.clone()
            assert torch.equal(out, first)


def test_layer_prefill_rejects_bad_arguments():
    with make_ctx(256, 4, 4, 64, 688, torch.float32, 128) as ctx:
        wl = iso_inputs.WORKLOADS["tiny_f32"]
        x, w = iso_inputs.make_workload_inputs(wl, seed=0)
        w_dev = {k: v.to(DEV) for k, v in w.items()}
        xd = x.to(DEV)
        kc = torch.zeros(128, 4, 64, device=DEV)
        for T, split, code in ((129, 0, iso.ISO_ERR_WORKSPACE), (128, 129, iso.ISO_ERR_SPLIT), (128, -1, iso.ISO_ERR_SPLIT),
                               (0, 0, iso.ISO_ERR_SHAPE)):
            with pytest.raises(iso.IsoError) as ei:
                ctx.layer_prefill(w_dev, xd, kc, kc.clone(), T, split)
            assert ei.value.code == code
        with pytest.raises(iso.IsoError) as ei:
            ctx.layer_prefill(w_dev, xd, kc, kc, 128, 64, comm=5)
        assert ei.value.code == iso.ISO_ERR_SHAPE


# ------------------------------------------------------------------------------ full-size workloads

def _sampled_parity(name, split, n_rows=64):
    wl = iso_inputs.WORKLOADS[name]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    rows = iso_inputs.sample_rows(wl.seq, split, n_rows, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_rows(f64(x), {k: f64(v) for k, v in w.items()}, sh, rows)
    w_dev = {k: v.to(DEV) for k, v in w.items()}
    errs = {}
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.torch_dtype, wl.seq) as ctx:
        for s in (0, split):
            out, kc, vc = run_layer(ctx, w_dev, x, wl.seq, s, wl.n_kv_heads, wl.head_dim, wl.seq, iso.ISO_COMM_D2H,
                                    poison=True)
            errs[s] = orc.max_rel_err(f64(out[rows]), ref["x_out"])
            assert errs[s] <= TOL_LAYER[wl.dtype], (name, s, errs[s])
            ek = orc.max_rel_err(f64(kc), ref["k_cache"])
            ev = orc.max_rel_err(f64(vc), ref["v_cache"])
            assert ek <= TOL_LAYER[wl.dtype] and ev <= TOL_LAYER[wl.dtype], (name, s, ek, ev)
            errs[(s, "kv")] = (ek, ev)
    print(name, "max_rel_err", errs)


def test_full_size_30b_tp4_2k_sampled_rows():
    _sampled_parity("30b_tp4_2k", 1024)


def test_full_size_70b_tp8_4k_sampled_rows():
    _sampled_parity("70b_tp8_4k", 2048)


@pytest.mark.parametrize("split", [4096, 4915, 5792])
def test_full_size_70b_tp4_8k_sampled_rows(split):
    _sampled_parity("70b_tp4_8k", split, n_rows=48)
