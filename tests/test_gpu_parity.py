"""GPU parity: every entry point of libiso against the CPU oracle on the same seeded inputs.

Tolerances (metric: max |got - ref| / max(|ref|, rms(ref)), see oracle.max_rel_err):
  fp32 path  : 1e-4 for the whole layer; single steps 2e-5 (fp32 accumulation over <= 1e3 terms).
  bf16 path  : 2e-2 for the whole layer.  Single steps: the output rounding alone is 2^-8 = 3.9e-3
               relative; steps that also round an intermediate (attention probabilities, SwiGLU input)
               get 1e-2.
"""
import numpy as np
import pytest

import paper_2409_11155_amd as iso      # first: binds libiso to the HIP runtime it was built against
import iso_inputs
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

TOL_LAYER = {"f32": 1e-4, "bf16": 2e-2}
TOL_STEP = {"f32": 2e-5, "bf16": 1e-2}
NAN_BYTE = 0xFF        # 0xFFFF (bf16) and 0xFFFFFFFF (fp32) are NaN bit patterns


def dev(a, dt):
    return iso.DeviceArray.from_numpy(a, dt)


def f64(buf):
    """float64 values of a DeviceArray (downloaded) or of a host storage array given its dtype."""
    return iso_inputs.to_f64(buf.numpy(), buf.dtype)


def h64(a, dt):
    return iso_inputs.to_f64(a, dt)


def shape_of(hidden, nq, nkv, d, ffn, eps=1e-6, base=10000.0):
    return orc.LayerShape(hidden, nq, nkv, d, ffn, eps, base)


def make_ctx(hidden, nq, nkv, d, ffn, dtype, max_seq, two_streams=True):
    cfg = iso.make_cfg(hidden, nq, nkv, d, ffn, dtype, max_seq)
    return iso.Context(cfg, two_streams=two_streams)


# ------------------------------------------------------------------------------ element-wise steps

@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("T,H", [(1, 256), (37, 1000), (130, 8192), (5, 16384)])
def test_rmsnorm_and_residual_rmsnorm(dt, T, H):
    x = iso_inputs.randn((T, H), seed=T * 7 + H, dtype=dt)
    delta = iso_inputs.randn((T, H), seed=T * 7 + H + 1, dtype=dt, scale=0.5)
    g = iso_inputs.store(1 + 0.1 * iso_inputs.bf16_bits_to_f32(iso_inputs.randn((H,), seed=H, dtype="bf16")), dt)
    with make_ctx(H, 4, 4, 64, 64, dt, 256) as ctx:
        xd, dd, gd = dev(x, dt), dev(delta, dt), dev(g, dt)
        y = iso.DeviceArray((T, H), dt)
        ctx.rmsnorm(xd, gd, y, T, ctx.stream0)
        ctx.sync()
        tol = TOL_STEP[dt]
        assert orc.max_rel_err(f64(y), orc.rmsnorm(h64(x, dt), h64(g, dt), 1e-6)) <= tol
        # fused: x += delta (in place), y = norm(x)
        y2 = iso.DeviceArray((T, H), dt)
        ctx.residual_rmsnorm(xd, dd, gd, y2, T, ctx.stream0)
        ctx.sync()
        x1 = h64(x, dt) + h64(delta, dt)
        assert orc.max_rel_err(f64(xd), x1) <= tol
        assert orc.max_rel_err(f64(y2), orc.rmsnorm(x1, h64(g, dt), 1e-6)) <= tol
        # residual only
        xd2 = dev(x, dt)
        ctx.residual_rmsnorm(xd2, dd, None, None, T, ctx.stream0)
        ctx.sync()
        assert orc.max_rel_err(f64(xd2), x1) <= tol


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("nq,nkv,d", [(4, 4, 64), (8, 1, 128), (13, 13, 128), (6, 2, 64)])
def test_rope_kv_write(dt, nq, nkv, d):
    Tc, q_offset, max_seq = 70, 41, 128
    qkv = iso_inputs.randn((Tc, (nq + 2 * nkv) * d), seed=nq * 100 + d, dtype=dt)
    seven = iso_inputs.store(np.full((max_seq, nkv, d), 7.0, dtype=np.float32), dt)
    with make_ctx(256, nq, nkv, d, 64, dt, max_seq) as ctx:
        qd, kc, vc = dev(qkv, dt), dev(seven, dt), dev(seven, dt)
        ctx.rope_kv_write(qd, kc, vc, Tc, q_offset, ctx.stream0)
        ctx.sync()
        pos = np.arange(q_offset, q_offset + Tc)
        ref = h64(qkv, dt)
        q_ref = orc.rope(ref[:, : nq * d].reshape(Tc, nq, d), pos, 10000.0)
        k_ref = orc.rope(ref[:, nq * d:(nq + nkv) * d].reshape(Tc, nkv, d), pos, 10000.0)
        v_ref = ref[:, (nq + nkv) * d:].reshape(Tc, nkv, d)
        tol = TOL_STEP[dt]
        kcn, vcn = f64(kc), f64(vc)
        assert orc.max_rel_err(f64(qd)[:, : nq * d].reshape(Tc, nq, d), q_ref) <= tol
        assert orc.max_rel_err(kcn[q_offset:q_offset + Tc], k_ref) <= tol
        np.testing.assert_array_equal(vcn[q_offset:q_offset + Tc], v_ref)       # v is a copy: bit-exact
        # rows outside the chunk are untouched
        assert np.all(kcn[:q_offset] == 7.0) and np.all(kcn[q_offset + Tc:] == 7.0)
        assert np.all(vcn[:q_offset] == 7.0) and np.all(vcn[q_offset + Tc:] == 7.0)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
@pytest.mark.parametrize("T,F", [(1, 8), (33, 688), (129, 3584)])
def test_swiglu(dt, T, F):
    gu = iso_inputs.randn((T, 2 * F), seed=F, dtype=dt, scale=2.0)
    with make_ctx(256, 4, 4, 64, F, dt, 256) as ctx:
        a = iso.DeviceArray((T, F), dt)
        ctx.swiglu(dev(gu, dt), a, T, ctx.stream0)
        ctx.sync()
        assert orc.max_rel_err(f64(a), orc.swiglu(h64(gu, dt))) <= TOL_STEP[dt]


# ------------------------------------------------------------------------------ projections

GEMM_SHAPES = [(1, 8, 8), (64, 128, 64), (128, 128, 64), (129, 130, 72), (300, 257, 1000), (77, 768, 256),
               (256, 384, 688), (513, 1280, 2048), (1000, 520, 1664), (260, 8, 64),
               # two, three and five k-slices: the ends of the direct-to-LDS pipeline (three W stages, two A stages)
               (200, 264, 128), (300, 520, 192), (70, 136, 320)]


@pytest.mark.parametrize("dt,flags", [("f32", 0), ("bf16", 0), ("bf16", iso.ISO_FLAG_GEMM_STAGED),
                                      ("bf16", iso.ISO_FLAG_SIMPLE_GEMM),
                                      ("bf16", 1 << 8), ("bf16", 2 << 8), ("bf16", 3 << 8), ("bf16", 4 << 8),
                                      ("bf16", 5 << 8), ("bf16", 6 << 8), ("bf16", 9 << 8)])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_rowpar(dt, flags, M, N, K):
    a = iso_inputs.randn((M, K), seed=M + N + K, dtype=dt)
    w = iso_inputs.randn((N, K), seed=M + N + K + 1, dtype=dt, scale=K ** -0.5)
    with make_ctx(256, 4, 4, 64, 64, dt, 256) as ctx:
        ctx.set_flags(flags)
        c = iso.DeviceArray((M, N), dt, fill_byte=0)
        sink = iso.PinnedArray((M, N), dt)
        sink.array[...] = 0
        ctx.gemm_rowpar(dev(a, dt), dev(w, dt), c, M, N, K, ctx.stream0, sink.ptr)
        ctx.sync()
        ref = orc.linear(h64(a, dt), h64(w, dt))
        assert orc.max_rel_err(f64(c), ref) <= TOL_STEP[dt]
        np.testing.assert_array_equal(sink.array, c.numpy())   # the communication stand-in moved exactly the partial
        sink.free()


def test_gemm_stream_k_repeated_launches_and_both_streams():
    """The stream-K kernel hands partial tiles between workgroups through a workspace whose flags are never
    reset (each launch has its own epoch): launches in a row, with changing shapes and on both streams of the
    context at once, must each match the oracle and the plain 256x256 kernel bit for bit in nothing but sum order
    (compared through the oracle, not to each other)."""
    dt = "bf16"
    with make_ctx(256, 4, 4, 64, 64, dt, 256) as ctx:
        ctx.set_flags(6 << 8)
        cases = [(700, 1000, 4096), (513, 1280, 2048), (256, 256, 64), (1024, 2304, 1664), (300, 520, 8192),
                 (700, 1000, 4096)]
        outs = []
        for i, (M, N, K) in enumerate(cases):
            a = iso_inputs.randn((M, K), seed=100 + i, dtype=dt)
            w = iso_inputs.randn((N, K), seed=200 + i, dtype=dt, scale=K ** -0.5)
            c = iso.DeviceArray((M, N), dt, fill_byte=NAN_BYTE)
            stream = ctx.stream0 if i % 2 == 0 else ctx.stream1
            ctx.gemm_rowpar(dev(a, dt), dev(w, dt), c, M, N, K, stream)
            outs.append((a, w, c))
        ctx.sync()
        for a, w, c in outs:
            assert orc.max_rel_err(f64(c), orc.linear(h64(a, dt), h64(w, dt))) <= TOL_STEP[dt]


def test_gemm_rejects_bad_shapes():
    with make_ctx(256, 4, 4, 64, 64, "bf16", 256) as ctx:
        a = iso.DeviceArray((4, 12), "bf16", fill_byte=0)
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
    (640, 384, 1024, 2, 1),      # many tiles, kv_len == max_seq
]


@pytest.mark.parametrize("dt,d,flags", [("f32", 64, 0), ("f32", 128, 0), ("bf16", 128, 0),
                                        ("bf16", 128, iso.ISO_FLAG_ATTN_STAGED),
                                        ("bf16", 128, iso.ISO_FLAG_SIMPLE_ATTN), ("bf16", 64, 0),
                                        # the three launch shapes of the direct-to-LDS kernel, forced (bits 12..13)
                                        ("bf16", 128, 1 << 12), ("bf16", 128, 2 << 12), ("bf16", 128, 3 << 12),
                                        # keys split across 2, 3 and 4 workgroups (bits 14..16), in each launch shape
                                        ("bf16", 128, (1 << 12) | (2 << 14)), ("bf16", 128, (1 << 12) | (4 << 14)),
                                        ("bf16", 128, (2 << 12) | (3 << 14)), ("bf16", 128, (3 << 12) | (2 << 14)),
                                        ("bf16", 128, (3 << 12) | (4 << 14)), ("bf16", 128, 1 << 14)])
@pytest.mark.parametrize("Tc,q_offset,kv_len,nq,nkv", ATTN_CASES)
def test_attn_chunk(dt, d, flags, Tc, q_offset, kv_len, nq, nkv):
    q, k, v = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=Tc + q_offset, dtype=dt)
    with make_ctx(256, nq, nkv, d, 64, dt, 1024) as ctx:
        ctx.set_flags(flags)
        out = iso.DeviceArray((Tc, nq * d), dt, fill_byte=0)
        ctx.attn_chunk(dev(q, dt), dev(k, dt), dev(v, dt), out, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        ref = orc.attention_chunk(h64(q, dt), h64(k, dt), h64(v, dt), q_offset, kv_len).reshape(Tc, nq * d)
        tol = TOL_STEP[dt]
        if flags >> 14:      # a launch that split the keys leaves its arrival counters at zero: run it once more
            out.fill(0)
            ctx.attn_chunk(dev(q, dt), dev(k, dt), dev(v, dt), out, Tc, q_offset, kv_len, ctx.stream0)
            ctx.sync()
        if dt == "bf16" and d == 128 and flags != iso.ISO_FLAG_SIMPLE_ATTN:
            # the matrix-core kernel rounds the probabilities to bf16 before the second product:
            # |d out| <= 2^-9 * sum_j p_j |v_j| <= 2^-9 max|v|, on top of the 2^-8 output rounding
            rms = float(np.sqrt(np.mean(ref * ref)))
            tol = 2.0 ** -9 * float(np.abs(h64(v, dt)).max()) / rms + 2.0 ** -8 + 1e-4
        err = orc.max_rel_err(f64(out), ref)
        assert err <= tol, (err, tol)


@pytest.mark.parametrize("Tc,q_offset,nq,nkv", [(2048, 1024, 32, 4), (1920, 0, 34, 2)])
def test_attn_chunk_mid_size_launch_takes_two_row_blocks_per_workgroup(Tc, q_offset, nq, nkv):
    """512 and more workgroups' worth of row blocks: the launch pairs the longest row block with the shortest
    (chosen by itself here, not forced); an odd block count leaves the middle one alone."""
    dt, d, kv_len = "bf16", 128, q_offset + Tc
    q, k, v = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=9, dtype=dt)
    with make_ctx(256, nq, nkv, d, 64, dt, kv_len) as ctx:
        out = iso.DeviceArray((Tc, nq * d), dt, fill_byte=NAN_BYTE)
        ctx.attn_chunk(dev(q, dt), dev(k, dt), dev(v, dt), out, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        ref = orc.attention_chunk(h64(q, dt), h64(k, dt), h64(v, dt), q_offset, kv_len).reshape(Tc, nq * d)
        rms = float(np.sqrt(np.mean(ref * ref)))
        tol = 2.0 ** -9 * float(np.abs(h64(v, dt)).max()) / rms + 2.0 ** -8 + 1e-4
        err = orc.max_rel_err(f64(out), ref)
        assert err <= tol, (err, tol)


@pytest.mark.parametrize("Tc,q_offset", [(53248, 77824), (77824, 0)])
def test_attn_chunk_full_size_deep_in_a_128k_cache_sampled_rows(Tc, q_offset):
    """Both chunks of the 128k prompt cut at 77824 (70B, TP=8: 8 query heads on 1 KV head) at their real size and in
    the launch shape the library picks for them (3328 and 4864 row blocks: one per workgroup, two workgroups per
    compute unit).  The oracle takes the sampled rows one query at a time."""
    dt, d, nq, nkv = "bf16", 128, 8, 1
    kv_len = q_offset + Tc
    q, k, v = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=128, dtype=dt)
    with make_ctx(256, nq, nkv, d, 64, dt, kv_len) as ctx:
        out = iso.DeviceArray((Tc, nq * d), dt, fill_byte=NAN_BYTE)
        ctx.attn_chunk(dev(q, dt), dev(k, dt), dev(v, dt), out, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        got = f64(out)
    assert np.isfinite(got).all()
    gen = np.random.default_rng(7)
    rows = sorted({0, 1, 127, 128, Tc - 129, Tc - 128, Tc - 1} | set(int(r) for r in gen.integers(0, Tc, 25)))
    k64, v64 = h64(k, dt), h64(v, dt)
    # A row averages ~1e5 values, so its output is small against max|v| and the worst-case bound of the short cases
    # (a multiple of max|v| / rms) says nothing here.  What the arithmetic gives, relative to the row's rms: the bf16
    # rounding of the output is at most 2^-8 of an element, hence 2^-8 max|ref| / rms; the bf16 rounding of the
    # probabilities puts independent relative errors of at most 2^-8 on the terms of a sum whose own root-mean-square
    # is the row's rms, i.e. a standard deviation of at most 2^-8 / sqrt(3) of it, six of which cover every compared
    # element.  (About 0.03 for a row whose largest element is 4 rms; gross for any indexing mistake at this size.)
    worst = 0.0
    for i in rows:
        ref = orc.attention_chunk(h64(q[i:i + 1], dt), k64, v64, q_offset + i, kv_len).reshape(nq * d)
        rms = float(np.sqrt(np.mean(ref * ref)))
        tol = 2.0 ** -8 * float(np.abs(ref).max()) / rms + 6.0 * 2.0 ** -8 / np.sqrt(3.0)
        err = float(np.abs(got[i] - ref).max() / rms)
        worst = max(worst, err / tol)
        assert err <= tol, (i, err, tol)
    print(f"deep-cache attention: worst row at {worst:.2f} of its bound over {len(rows)} rows")


@pytest.mark.parametrize("Tc,q_offset,nq,nkv", [(1024, 0, 13, 13), (1024, 1024, 13, 13), (2048, 2048, 8, 1),
                                                 (1000, 1500, 6, 2)])
def test_attn_chunk_small_launch_splits_keys_across_workgroups(Tc, q_offset, nq, nkv):
    """Chunks of 1k-2k rows give about a hundred row-block workgroups on 256 compute units: the launch rule then
    splits every row block's keys over several workgroups (chosen by itself here, not forced), each parks a partial
    state and the last arriver folds them in share order.  All rows against the oracle, on both streams of the
    context at once (each stream has its own workspace), and twice: the second launch finds the counters at zero and
    must give the same bits as the first (the fold order is fixed, whoever arrives last)."""
    dt, d, kv_len = "bf16", 128, q_offset + Tc
    q, k, v = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=Tc + nq, dtype=dt)
    ref = orc.attention_chunk(h64(q, dt), h64(k, dt), h64(v, dt), q_offset, kv_len).reshape(Tc, nq * d)
    rms = float(np.sqrt(np.mean(ref * ref)))
    tol = 2.0 ** -9 * float(np.abs(h64(v, dt)).max()) / rms + 2.0 ** -8 + 1e-4
    with make_ctx(256, nq, nkv, d, 64, dt, kv_len) as ctx:
        qd, kd, vd = dev(q, dt), dev(k, dt), dev(v, dt)
        outs = [iso.DeviceArray((Tc, nq * d), dt, fill_byte=NAN_BYTE) for _ in range(4)]
        for i, o in enumerate(outs):
            ctx.attn_chunk(qd, kd, vd, o, Tc, q_offset, kv_len, ctx.stream0 if i % 2 == 0 else ctx.stream1)
        ctx.sync()
        first = outs[0].numpy()
        err = orc.max_rel_err(h64(first, dt), ref)
        assert err <= tol, (err, tol)
        for o in outs[1:]:
            np.testing.assert_array_equal(o.numpy(), first)
        # the same launch with the split switched off agrees within the bound as well (other sum order)
        ctx.set_flags(1 << 14)
        plain = iso.DeviceArray((Tc, nq * d), dt, fill_byte=NAN_BYTE)
        ctx.attn_chunk(qd, kd, vd, plain, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        assert orc.max_rel_err(f64(plain), ref) <= tol


def test_attn_chunk_rejects_bad_arguments():
    with make_ctx(256, 4, 4, 64, 64, "f32", 64) as ctx:
        t = iso.DeviceArray((64, 256), "f32", fill_byte=0)
        for args, code in (((0, 0, 1), iso.ISO_ERR_SHAPE), ((4, -1, 4), iso.ISO_ERR_SHAPE), ((4, 0, 0), iso.ISO_ERR_SHAPE),
                           ((4, 0, 65), iso.ISO_ERR_WORKSPACE), ((65, 0, 4), iso.ISO_ERR_WORKSPACE)):
            with pytest.raises(iso.IsoError) as ei:
                ctx.attn_chunk(t, t, t, t, *args, ctx.stream0)
            assert ei.value.code == code


# ------------------------------------------------------------------------------ whole layer

def run_layer(ctx, w_dev, x_host, dt, T, split, nkv, d, max_seq, comm=iso.ISO_COMM_NONE, sched=iso.ISO_SCHED_OVERLAP,
              poison=False):
    x = dev(x_host, dt)
    kc = iso.DeviceArray((max_seq, nkv, d), dt, fill_byte=NAN_BYTE if poison else 0)
    vc = iso.DeviceArray((max_seq, nkv, d), dt, fill_byte=NAN_BYTE if poison else 0)
    ctx.layer_prefill(w_dev, x, kc, vc, T, split, comm, sched)
    ctx.sync()
    return x, kc, vc


def oracle_weights(w, dt):
    return {k: h64(v, dt) for k, v in w.items()}


def test_tiny_f32_layer_unsplit_and_every_tested_split():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_unsplit(h64(x, "f32"), oracle_weights(w, "f32"), sh)
    w_dev = iso.upload_weights(w, "f32")
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, "f32", wl.seq) as ctx:
        for split in (0, wl.seq, 64, 1, 127, 33, 77, 100):
            for sched in (iso.ISO_SCHED_OVERLAP, iso.ISO_SCHED_SERIAL):
                for comm in (iso.ISO_COMM_NONE, iso.ISO_COMM_D2H):
                    out, kc, vc = run_layer(ctx, w_dev, x, "f32", wl.seq, split, wl.n_kv_heads, wl.head_dim, wl.seq,
                                            comm, sched, poison=True)
                    err = orc.max_rel_err(f64(out), ref["x_out"])
                    assert err <= TOL_LAYER["f32"], (split, sched, comm, err)
                    assert orc.max_rel_err(f64(kc), ref["k_cache"]) <= TOL_STEP["f32"]
                    assert orc.max_rel_err(f64(vc), ref["v_cache"]) <= TOL_STEP["f32"]


def test_tiny_f32_layer_matches_the_oracles_iso_path_too():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_iso(h64(x, "f32"), oracle_weights(w, "f32"), sh, wl.split)
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, "f32", wl.seq) as ctx:
        out, _, _ = run_layer(ctx, iso.upload_weights(w, "f32"), x, "f32", wl.seq, wl.split, wl.n_kv_heads,
                              wl.head_dim, wl.seq)
        assert orc.max_rel_err(f64(out), ref["x_out"]) <= TOL_LAYER["f32"]


def test_comm_stand_in_delivers_both_partials_to_the_host():
    """With ISO_COMM_D2H the pinned sink holds the o_proj partial and the down partial of every token: check
    them against the oracle's intermediates (x1 - x and x_out - x1)."""
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_unsplit(h64(x, "f32"), oracle_weights(w, "f32"), sh)
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, "f32", wl.seq) as ctx:
        run_layer(ctx, iso.upload_weights(w, "f32"), x, "f32", wl.seq, wl.split, wl.n_kv_heads, wl.head_dim, wl.seq,
                  iso.ISO_COMM_D2H)
        import ctypes
        n = wl.seq * wl.hidden
        sink = np.frombuffer((ctypes.c_float * (2 * n)).from_address(ctx.host_sink()), dtype=np.float32).copy()
        pa, pm = sink[:n].reshape(wl.seq, wl.hidden), sink[n:].reshape(wl.seq, wl.hidden)
        assert orc.max_rel_err(pa, ref["x1"] - h64(x, "f32")) <= TOL_LAYER["f32"]
        assert orc.max_rel_err(pm, ref["x_out"] - ref["x1"]) <= TOL_LAYER["f32"]


@pytest.mark.parametrize("flags", [0, iso.ISO_FLAG_SIMPLE_GEMM | iso.ISO_FLAG_SIMPLE_ATTN, iso.ISO_FLAG_GEMM_STAGED,
                                   iso.ISO_FLAG_NO_FUSE, 1 << 8, 2 << 8, 3 << 8, 4 << 8, 6 << 8])
@pytest.mark.parametrize("hidden,nq,nkv,ffn,T,splits", [
    (512, 4, 1, 768, 300, (0, 130, 299)),       # GQA, ragged everything
    (384, 3, 3, 200, 257, (128, 1)),            # MHA, odd head count
    (128, 2, 1, 192, 260, (0, 100)),            # two and three k-slices in the projections
])
def test_small_bf16_layer_all_rows(flags, hidden, nq, nkv, ffn, T, splits):
    d, dt = 128, "bf16"
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=11, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=11, dtype=dt)
    ref = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), shape_of(hidden, nq, nkv, d, ffn))
    w_dev = iso.upload_weights(w, dt)
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 320) as ctx:
        ctx.set_flags(flags)
        for split in splits:
            out, kc, vc = run_layer(ctx, w_dev, x, dt, T, split, nkv, d, 320, iso.ISO_COMM_D2H, poison=True)
            err = orc.max_rel_err(f64(out), ref["x_out"])
            assert err <= TOL_LAYER["bf16"], (split, err)
            # cached K went through three bf16 roundings (norm output, projection output, rotation)
            assert orc.max_rel_err(f64(kc)[:T], ref["k_cache"]) <= TOL_LAYER["bf16"]
            assert orc.max_rel_err(f64(vc)[:T], ref["v_cache"]) <= TOL_LAYER["bf16"]


@pytest.mark.parametrize("variant", [1 << 8, 6 << 8, 0])
@pytest.mark.parametrize("hidden,nq,nkv,T,split", [(512, 4, 1, 300, 130), (384, 3, 3, 700, 257), (1024, 8, 2, 1100, 0)])
def test_rotary_and_cache_write_in_the_qkv_epilogue_against_the_separate_kernel(variant, hidden, nq, nkv, T, split):
    """bf16 layers with head_dim 128 rotate q/k and write the caches in the epilogue of the QKV projection (256-wide
    tile, forced here as variant 1, and its stream-K launch, variant 6; 0 = the launch rule's own choice).  Against
    the same layer with the separate rotary kernel (ISO_FLAG_NO_FUSE): V rows are copies of the same bf16
    projection output and must be the same bits; K rows and the layer output go through the same roundings (bf16
    projection output, rotation in fp32, bf16) and must both match the oracle, the fused K as closely as the other."""
    d, dt, ffn = 128, "bf16", 512
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=23, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=23, dtype=dt)
    ref = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), shape_of(hidden, nq, nkv, d, ffn))
    w_dev = iso.upload_weights(w, dt)
    max_seq = T + 37                                   # rows past the prompt must stay untouched
    with make_ctx(hidden, nq, nkv, d, ffn, dt, max_seq) as ctx:
        got = {}
        for name, flags in (("fused", variant), ("separate", variant | iso.ISO_FLAG_NO_FUSE)):
            ctx.set_flags(flags)
            ctx.timing_enable(True)
            out, kc, vc = run_layer(ctx, w_dev, x, dt, T, split, nkv, d, max_seq, iso.ISO_COMM_D2H, poison=True)
            n_rope = ctx.timing_read()["rope_kv"][1]
            ctx.timing_enable(False)
            got[name] = (f64(out), f64(kc), vc.numpy(), n_rope)
            assert orc.max_rel_err(got[name][0], ref["x_out"]) <= TOL_LAYER[dt], name
            assert orc.max_rel_err(got[name][1][:T], ref["k_cache"]) <= TOL_LAYER[dt], name
            assert np.isnan(got[name][1][T:]).all(), name
        n_chunks = 2 if 0 < split < T else 1
        assert got["separate"][3] == n_chunks
        if variant:                                    # forced onto a head-owning kernel: no rotary launch left
            assert got["fused"][3] == 0
        np.testing.assert_array_equal(got["fused"][2], got["separate"][2])
        rms_f = np.sqrt(np.mean((got["fused"][1][:T] - ref["k_cache"]) ** 2))
        rms_s = np.sqrt(np.mean((got["separate"][1][:T] - ref["k_cache"]) ** 2))
        assert rms_f <= rms_s * 1.02, (rms_f, rms_s)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_degenerate_prompts_of_one_two_and_three_tokens(dt):
    """The shortest prompts: a single token attends to itself only; with two or three tokens every cut leaves
    one-token chunks."""
    hidden, nq, nkv, d, ffn = 256, 4, 2, 64, 256
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=31, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    w_dev = iso.upload_weights(w, dt)
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 8) as ctx:
        for T in (1, 2, 3):
            x = iso_inputs.make_hidden(T, hidden, seed=31 + T, dtype=dt)
            ref = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), sh)
            for split in range(0, T + 1):
                out, kc, vc = run_layer(ctx, w_dev, x, dt, T, split, nkv, d, 8, iso.ISO_COMM_D2H, poison=True)
                assert orc.max_rel_err(f64(out), ref["x_out"]) <= TOL_LAYER[dt], (T, split)
                assert orc.max_rel_err(f64(kc)[:T], ref["k_cache"]) <= TOL_LAYER[dt]
                assert np.isnan(f64(kc)[T:]).all()           # rows beyond the prompt are never written


def test_small_bf16_layer_with_head_dim_64():
    """head_dim 64 takes the one-wave-per-row attention kernel inside an otherwise matrix-core layer."""
    hidden, nq, nkv, d, ffn, T, dt = 512, 8, 2, 64, 640, 200, "bf16"
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=17, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=17, dtype=dt)
    ref = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), shape_of(hidden, nq, nkv, d, ffn))
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 256) as ctx:
        for split in (0, 77):
            out, kc, vc = run_layer(ctx, iso.upload_weights(w, dt), x, dt, T, split, nkv, d, 256, iso.ISO_COMM_D2H, poison=True)
            assert orc.max_rel_err(f64(out), ref["x_out"]) <= TOL_LAYER[dt], split
            assert orc.max_rel_err(f64(vc)[:T], ref["v_cache"]) <= TOL_LAYER[dt]


def test_two_layer_stack_equals_two_oracle_layers():
    hidden, nq, nkv, d, ffn, T, split, dt = 256, 2, 1, 128, 256, 200, 90, "bf16"
    layers = [iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=20 + l, dtype=dt) for l in range(2)]
    x = iso_inputs.make_hidden(T, hidden, seed=5, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    ref = h64(x, dt)
    for w in layers:
        ref = orc.layer_unsplit(ref, oracle_weights(w, dt), sh)["x_out"]
    layers_dev = [iso.upload_weights(w, dt) for w in layers]
    with make_ctx(hidden, nq, nkv, d, ffn, dt, T) as ctx:
        for s in (0, split):
            xd = dev(x, dt)
            kcs = iso.DeviceArray((2, T, nkv, d), dt, fill_byte=NAN_BYTE)
            vcs = iso.DeviceArray((2, T, nkv, d), dt, fill_byte=NAN_BYTE)
            ctx.stack_prefill(layers_dev, xd, kcs, vcs, T, s, iso.ISO_COMM_D2H)
            ctx.sync()
            # two layers compound the per-layer bf16 error: allow twice the per-layer bound
            assert orc.max_rel_err(f64(xd), ref) <= 2 * TOL_LAYER["bf16"]


@pytest.mark.parametrize("dt,hidden", [("bf16", 8256), ("f32", 4224)])
def test_two_layer_stack_with_rows_longer_than_the_norm_kernels_register_cache(dt, hidden):
    """Rows beyond 256 threads x 4 cached 16-byte pieces (8192 bf16 / 4096 fp32 elements) take the norm kernels'
    second loops: the mid-layer norm rebuilds x + attention partial there from its inputs, the kernel that closes a
    layer re-reads the row it has just written in place."""
    nq, nkv, d, ffn, T, split = 2, 1, 128, 256, 70, 33
    layers = [iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=60 + l, dtype=dt) for l in range(2)]
    x = iso_inputs.make_hidden(T, hidden, seed=6, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    ref = h64(x, dt)
    for w in layers:
        ref = orc.layer_unsplit(ref, oracle_weights(w, dt), sh)["x_out"]
    layers_dev = [iso.upload_weights(w, dt) for w in layers]
    with make_ctx(hidden, nq, nkv, d, ffn, dt, T) as ctx:
        for s in (0, split):
            xd = dev(x, dt)
            kcs = iso.DeviceArray((2, T, nkv, d), dt, fill_byte=NAN_BYTE)
            vcs = iso.DeviceArray((2, T, nkv, d), dt, fill_byte=NAN_BYTE)
            ctx.stack_prefill(layers_dev, xd, kcs, vcs, T, s, iso.ISO_COMM_D2H)
            ctx.sync()
            err = orc.max_rel_err(f64(xd), ref)
            assert err <= 2 * TOL_LAYER[dt], (s, err)


def test_kv_event_orders_the_chunks_and_runs_are_bit_identical():
    """Chunk 1 must not read the cache before chunk 0 wrote it (Section 3.1).  The cache starts as NaN, so a
    read that overtook the write would surface as NaN; repeated runs must also agree bit for bit."""
    hidden, nq, nkv, d, ffn, T, split, dt = 1024, 8, 1, 128, 1024, 1024, 512, "bf16"
    w = iso.upload_weights(iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=3, dtype=dt), dt)
    x = iso_inputs.make_hidden(T, hidden, seed=3, dtype=dt)
    with make_ctx(hidden, nq, nkv, d, ffn, dt, T) as ctx:
        first = None
        for _ in range(10):
            out, _, _ = run_layer(ctx, w, x, dt, T, split, nkv, d, T, iso.ISO_COMM_D2H, poison=True)
            bits = out.numpy()
            assert not np.isnan(iso_inputs.bf16_bits_to_f32(bits)).any()
            if first is None:
                first = bits
            np.testing.assert_array_equal(bits, first)


def test_layer_prefill_rejects_bad_arguments():
    with make_ctx(256, 4, 4, 64, 688, "f32", 128) as ctx:
        wl = iso_inputs.WORKLOADS["tiny_f32"]
        x, w = iso_inputs.make_workload_inputs(wl, seed=0)
        w_dev = iso.upload_weights(w, "f32")
        xd = dev(x, "f32")
        kc = iso.DeviceArray((128, 4, 64), "f32", fill_byte=0)
        vc = iso.DeviceArray((128, 4, 64), "f32", fill_byte=0)
        for T, split, code in ((129, 0, iso.ISO_ERR_WORKSPACE), (128, 129, iso.ISO_ERR_SPLIT), (128, -1, iso.ISO_ERR_SPLIT),
                               (0, 0, iso.ISO_ERR_SHAPE)):
            with pytest.raises(iso.IsoError) as ei:
                ctx.layer_prefill(w_dev, xd, kc, vc, T, split)
            assert ei.value.code == code
        with pytest.raises(iso.IsoError) as ei:
            ctx.layer_prefill(w_dev, xd, kc, vc, 128, 64, comm=5)
        assert ei.value.code == iso.ISO_ERR_SHAPE


# ------------------------------------------------------------------------------ full-size workloads

def _sampled_parity(name, split, n_rows=64):
    wl = iso_inputs.WORKLOADS[name]
    dt = wl.dtype
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    rows = iso_inputs.sample_rows(wl.seq, split, n_rows, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_rows(h64(x, dt), oracle_weights(w, dt), sh, rows)
    w_dev = iso.upload_weights(w, dt)
    errs = {}
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, dt, wl.seq) as ctx:
        for s in (0, split):
            out, kc, vc = run_layer(ctx, w_dev, x, dt, wl.seq, s, wl.n_kv_heads, wl.head_dim, wl.seq, iso.ISO_COMM_D2H,
                                    poison=True)
            errs[s] = orc.max_rel_err(f64(out)[rows], ref["x_out"])
            assert errs[s] <= TOL_LAYER[dt], (name, s, errs[s])
            ek = orc.max_rel_err(f64(kc), ref["k_cache"])
            ev = orc.max_rel_err(f64(vc), ref["v_cache"])
            assert ek <= TOL_LAYER[dt] and ev <= TOL_LAYER[dt], (name, s, ek, ev)
            errs[(s, "kv")] = (ek, ev)
    print(name, "max_rel_err", errs)


def test_full_size_30b_tp4_2k_sampled_rows():
    _sampled_parity("30b_tp4_2k", 1024)


def test_full_size_70b_tp8_4k_sampled_rows():
    _sampled_parity("70b_tp8_4k", 2048)


@pytest.mark.parametrize("split", [4096, 4915, 5792])
def test_full_size_70b_tp4_8k_sampled_rows(split):
    _sampled_parity("70b_tp4_8k", split, n_rows=48)


def test_full_size_70b_tp8_32k_long_prompt_sampled_rows():
    """Long prompt of the paper's Table 1: attention over 32k keys is a quarter of the layer's flops."""
    _sampled_parity("70b_tp8_32k", 18432, n_rows=32)


def test_stack_at_70b_tp8_16k_shape_layer_by_layer():
    """Three layers of the 80-layer 70B TP=8 stack shape at the full 16k prompt, split 8192/8192, chunks kept on
    their streams across layers.  The bf16 bound is per layer, so each layer is checked from the GPU's own input
    to that layer: the l-layer stack output is the oracle's input for layer l (sampled rows, plus all K/V rows)."""
    wl = iso_inputs.WORKLOADS["70b_tp8_16k_stack"]
    dt, T, split, L = wl.dtype, wl.seq, wl.split, 3
    layers = [iso_inputs.make_layer(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, seed=1000 + l, dtype=dt)
              for l in range(L)]
    x0 = iso_inputs.make_hidden(T, wl.hidden, seed=0, dtype=dt)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    rows = iso_inputs.sample_rows(T, split, 24, seed=2)
    layers_dev = [iso.upload_weights(w, dt) for w in layers]
    errs = []
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, dt, T) as ctx:
        outs = []
        for n in range(1, L + 1):           # n-layer stacks from the same input: outs[n-1] = input of layer n
            xd = dev(x0, dt)
            kcs = iso.DeviceArray((n, T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
            vcs = iso.DeviceArray((n, T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
            ctx.stack_prefill(layers_dev[:n], xd, kcs, vcs, T, split, iso.ISO_COMM_D2H)
            ctx.sync()
            outs.append(xd.numpy())
            if n == L:
                k_all, v_all = kcs.numpy(), vcs.numpy()
        # the single-layer entry point must agree bit for bit with a one-layer stack
        xd = dev(x0, dt)
        kc = iso.DeviceArray((T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
        vc = iso.DeviceArray((T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
        ctx.layer_prefill(layers_dev[0], xd, kc, vc, T, split, iso.ISO_COMM_D2H)
        ctx.sync()
        np.testing.assert_array_equal(xd.numpy(), outs[0])
    inputs = [x0] + outs[:-1]
    for l in range(L):
        ref = orc.layer_rows(h64(inputs[l], dt), oracle_weights(layers[l], dt), sh, rows)
        err = orc.max_rel_err(h64(outs[l], dt)[rows], ref["x_out"])
        ek = orc.max_rel_err(h64(k_all[l], dt), ref["k_cache"])
        ev = orc.max_rel_err(h64(v_all[l], dt), ref["v_cache"])
        errs.append((err, ek, ev))
        assert err <= TOL_LAYER[dt] and ek <= TOL_LAYER[dt] and ev <= TOL_LAYER[dt], (l, err, ek, ev)
    print("70b_tp8_16k_stack per-layer max_rel_err (x_out, k, v):", errs)


# ------------------------------------------------------------------------------ int8 payload (Section 3.2)

def _int8_bound(ref, w64, sh, dt):
    """Extra error the int8 payload may add on top of the layer bound: where the GPU's partial and the oracle's
    differ by rounding noise across a .5 boundary they take neighbouring codes, i.e. differ by one step
    (scale = row max / 127) at that element, once per communication point."""
    pm = orc.mlp_partial(ref["x1"], w64, sh)
    step = np.abs(ref["pa"]).max(axis=1) / 127.0 + np.abs(pm).max(axis=1) / 127.0
    rms = float(np.sqrt(np.mean(ref["x_out"] ** 2)))
    return float(step.max()) / rms, pm


def _check_sink_codes(ctx, T, H, pa, pm, dt, rows=None):
    """The pinned sink holds rows of H int8 codes + fp32 scale (pitch H + 16) for both points."""
    import ctypes
    e = 2 if dt == "bf16" else 4
    region = ctx.cfg.max_seq * H * e
    raw = np.frombuffer((ctypes.c_ubyte * (2 * region)).from_address(ctx.host_sink()), dtype=np.uint8)
    for which, part in ((0, pa), (1, pm)):
        blk = raw[which * region: which * region + T * (H + 16)].reshape(T, H + 16)
        codes = blk[:, :H].view(np.int8)
        scales = blk[:, H:H + 4].copy().view(np.float32)[:, 0]
        if rows is not None:
            codes, scales = codes[rows], scales[rows]
        ref_codes, ref_scales = orc.quantize_rows(part)
        tol_s = 1e-3 if dt == "f32" else 2e-2     # a code flip at the first point shifts the second partial a little
        np.testing.assert_allclose(scales, ref_scales, rtol=tol_s)
        d = np.abs(codes.astype(np.int32) - ref_codes.astype(np.int32))
        lim = 1 if dt == "f32" else 2           # bf16 partials carry ~1 % noise: up to ~1.3 codes at |code| = 127
        assert d.max() <= lim, d.max()
        if dt == "f32":
            assert np.mean(d > 0) < 0.01


def test_tiny_f32_layer_int8_payload():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    w64 = oracle_weights(w, "f32")
    ref = orc.layer_unsplit(h64(x, "f32"), w64, sh, quant=True)
    extra, pm = _int8_bound(ref, w64, sh, "f32")
    w_dev = iso.upload_weights(w, "f32")
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, "f32", wl.seq) as ctx:
        for split in (0, 64, 37):
            for sched in (iso.ISO_SCHED_OVERLAP, iso.ISO_SCHED_SERIAL):
                out, _, _ = run_layer(ctx, w_dev, x, "f32", wl.seq, split, wl.n_kv_heads, wl.head_dim, wl.seq,
                                      iso.ISO_COMM_D2H_INT8, sched, poison=True)
                got = f64(out)
                err = orc.max_rel_err(got, ref["x_out"])
                assert err <= TOL_LAYER["f32"] + extra, (split, err, extra)
                # away from code flips the result is as tight as without the payload
                close = np.abs(got - ref["x_out"]) <= 1e-4 * np.maximum(np.abs(ref["x_out"]), 1.0)
                assert close.mean() > 0.99
                _check_sink_codes(ctx, wl.seq, wl.hidden, ref["pa"], pm, "f32")


def test_small_bf16_layer_int8_payload():
    hidden, nq, nkv, d, ffn, T, dt = 512, 4, 1, 128, 768, 300, "bf16"
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=11, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=11, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    w64 = oracle_weights(w, dt)
    ref = orc.layer_unsplit(h64(x, dt), w64, sh, quant=True)
    extra, pm = _int8_bound(ref, w64, sh, dt)
    w_dev = iso.upload_weights(w, dt)
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 320) as ctx:
        for split in (0, 130):
            out, _, _ = run_layer(ctx, w_dev, x, dt, T, split, nkv, d, 320, iso.ISO_COMM_D2H_INT8, poison=True)
            err = orc.max_rel_err(f64(out), ref["x_out"])
            assert err <= TOL_LAYER["bf16"] + extra, (split, err, extra)
            _check_sink_codes(ctx, T, hidden, ref["pa"], pm, dt)


@pytest.mark.parametrize("name", ["30b_tp4_2k", "70b_tp8_4k"])
def test_full_size_int8_payload_sampled_rows(name):
    wl = iso_inputs.WORKLOADS[name]
    dt = wl.dtype
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    rows = iso_inputs.sample_rows(wl.seq, wl.split, 64, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    w64 = oracle_weights(w, dt)
    ref = orc.layer_rows(h64(x, dt), w64, sh, rows, quant=True)
    extra, pm = _int8_bound(ref, w64, sh, dt)
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, dt, wl.seq) as ctx:
        out, _, _ = run_layer(ctx, iso.upload_weights(w, dt), x, dt, wl.seq, wl.split, wl.n_kv_heads, wl.head_dim,
                              wl.seq, iso.ISO_COMM_D2H_INT8, poison=True)
        err = orc.max_rel_err(f64(out)[rows], ref["x_out"])
        print(name, "int8 payload: max_rel_err", err, "bound", TOL_LAYER[dt] + extra)
        assert err <= TOL_LAYER[dt] + extra
        _check_sink_codes(ctx, wl.seq, wl.hidden, ref["pa"], pm, dt, rows=rows)
