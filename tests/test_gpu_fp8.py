"""GPU parity of the FP8 (E4M3) projections: the row quantiser bit for bit, the FP8 GEMM against the oracle's product
of the same quantised operands, and the layer with ISO_FLAG_FP8_GEMM against the oracle's FP8 layer."""
import numpy as np
import pytest

import paper_2409_11155_amd as iso      # first: binds libiso to the HIP runtime it was built against
import iso_inputs
from oracle import iso_oracle as orc
from test_gpu_parity import (NAN_BYTE, TOL_LAYER, TOL_STEP, dev, f64, h64, make_ctx, oracle_weights, shape_of)

pytestmark = pytest.mark.gpu

# Layer bounds with FP8 projections.  The quantiser is checked bit for bit and the FP8 GEMM to the bf16 step bound
# on identical inputs (below); at layer level device and oracle quantise activations that differ by the bf16
# roundings of the device's intermediate tensors (2^-9 relative).  A fraction ~2^-9 / 2^-3.5 of the elements then
# lands on the other side of an FP8 rounding boundary and moves by one FP8 step (~2^-3.5 of the element), which
# perturbs a projection output by about sqrt(2^-5.5) * 2^-3.5 = 1.3e-2 of its rms (a numpy emulation of the device
# pipeline gives 1.26e-2 per projection and 2.1e-2 for the layer).  Four projections in quadrature, with margin:
TOL_RMS_FP8 = 3e-2
# The layer metric is a maximum over 1e5..1e7 elements; for errors that are sums of a few one-step flips the maximum
# sits 6-7 rms above zero (emulation: 6.7), so the bound on max_rel_err is
TOL_LAYER_FP8 = 0.2


def rms_rel_err(got, ref):
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.sqrt(np.mean((got - ref) ** 2) / np.mean(ref ** 2)))


def test_row_quantiser_matches_the_oracle_bit_for_bit():
    dt = "bf16"
    rows, cols = 37, 1000
    a = iso_inputs.randn((rows, cols), seed=21, dtype=dt)
    a32 = iso_inputs.bf16_bits_to_f32(a)
    a32[3] = 0.0                                   # all-zero row
    a32[5] *= 1e-20                                # tiny row: the scale carries the magnitude
    a32[7] *= 1e20
    a32[9, 1:] = 0.0                               # a single non-zero element maps to +-448
    a = iso_inputs.f32_to_bf16_bits(a32)
    want_v, want_s = orc.quantize_rows_fp8(h64(a, dt))
    with make_ctx(256, 4, 4, 64, 64, dt, 256) as ctx:
        q = iso.DeviceArray((rows, cols), "u8", fill_byte=0x7F)
        s = iso.DeviceArray((rows,), "f32")
        ctx.quantize_rows_fp8(dev(a, dt), rows, cols, q, s, ctx.stream0)
        ctx.sync()
        got_v = orc.fp8_e4m3_decode(q.numpy())
        assert not np.isnan(got_v).any()
        np.testing.assert_array_equal(got_v, want_v)
        np.testing.assert_array_equal(s.numpy().astype(np.float64), want_s)


FP8_GEMM_SHAPES = [(1, 8, 128), (128, 128, 128), (129, 136, 256), (300, 264, 1024), (513, 1280, 2048), (77, 768, 384),
                   (1024, 4992, 6656), (260, 8, 128)]


@pytest.mark.parametrize("flags", [0, 6 << 8])          # 6 << 8: the stream-K launch, forced
@pytest.mark.parametrize("M,N,K", FP8_GEMM_SHAPES)
def test_gemm_fp8(M, N, K, flags):
    dt = "bf16"
    a = iso_inputs.randn((M, K), seed=M + N + K, dtype=dt)
    w = iso_inputs.randn((N, K), seed=M + N + K + 1, dtype=dt, scale=K ** -0.5)
    with make_ctx(256, 4, 4, 64, 64, dt, 256) as ctx:
        ctx.set_flags(flags)
        a8, sa = iso.DeviceArray((M, K), "u8"), iso.DeviceArray((M,), "f32")
        w8, sw = iso.DeviceArray((N, K), "u8"), iso.DeviceArray((N,), "f32")
        ctx.quantize_rows_fp8(dev(a, dt), M, K, a8, sa, ctx.stream0)
        ctx.quantize_rows_fp8(dev(w, dt), N, K, w8, sw, ctx.stream0)
        c = iso.DeviceArray((M, N), dt, fill_byte=NAN_BYTE)
        for _ in range(3 if flags else 1):                 # stream-K: the workspace flags carry over between launches
            ctx.gemm_fp8(a8, sa, w8, sw, c, M, N, K, ctx.stream0)
        ctx.sync()
        ref = orc.linear_fp8(h64(a, dt), h64(w, dt))       # same inputs, same quantiser: only rounding order differs
        assert orc.max_rel_err(f64(c), ref) <= TOL_STEP[dt]


def test_fp8_entry_points_reject_bad_arguments():
    with make_ctx(256, 4, 4, 64, 64, "bf16", 256) as ctx:
        a8, s = iso.DeviceArray((8, 128), "u8", fill_byte=0), iso.DeviceArray((8,), "f32", fill_byte=0)
        c = iso.DeviceArray((8, 8), "bf16", fill_byte=0)
        for (M, N, K) in ((8, 8, 64), (8, 12, 128), (0, 8, 128)):
            with pytest.raises(iso.IsoError) as ei:
                ctx.gemm_fp8(a8, s, a8, s, c, M, N, K, ctx.stream0)
            assert ei.value.code == iso.ISO_ERR_SHAPE
        with pytest.raises(iso.IsoError) as ei:
            ctx.quantize_rows_fp8(c, 8, 12, a8, s, ctx.stream0)
        assert ei.value.code == iso.ISO_ERR_SHAPE
    with make_ctx(256, 4, 4, 64, 64, "f32", 256) as ctx:
        with pytest.raises(iso.IsoError) as ei:
            ctx.gemm_fp8(a8, s, a8, s, c, 8, 8, 128, ctx.stream0)
        assert ei.value.code == iso.ISO_ERR_DTYPE


@pytest.mark.parametrize("sk", [0, 6 << 8])             # 6 << 8: every projection through the stream-K launch
@pytest.mark.parametrize("hidden,nq,nkv,ffn,T,splits", [
    (512, 4, 1, 768, 300, (0, 130)),        # GQA, ragged rows
    (384, 3, 3, 256, 257, (128,)),          # MHA, odd head count
])
def test_small_bf16_layer_with_fp8_projections(hidden, nq, nkv, ffn, T, splits, sk):
    d, dt = 128, "bf16"
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=12, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=12, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    ref = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), sh, fp8=True)
    exact = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), sh)
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 320) as ctx:
        w_dev = ctx.add_fp8_weights(iso.upload_weights(w, dt))
        ctx.set_flags(iso.ISO_FLAG_FP8_GEMM | sk)
        for split in splits:
            xd = dev(x, dt)
            kc = iso.DeviceArray((320, nkv, d), dt, fill_byte=NAN_BYTE)
            vc = iso.DeviceArray((320, nkv, d), dt, fill_byte=NAN_BYTE)
            ctx.layer_prefill(w_dev, xd, kc, vc, T, split, iso.ISO_COMM_D2H)
            ctx.sync()
            err = orc.max_rel_err(f64(xd), ref["x_out"])
            assert err <= TOL_LAYER_FP8, (split, err)
            assert rms_rel_err(f64(xd), ref["x_out"]) <= TOL_RMS_FP8
            assert orc.max_rel_err(f64(kc)[:T], ref["k_cache"]) <= TOL_LAYER_FP8
            assert rms_rel_err(f64(kc)[:T], ref["k_cache"]) <= TOL_RMS_FP8
            # and the FP8 path really ran: the result is further from the exact layer than the bf16 path ever is
            assert orc.max_rel_err(f64(xd), exact["x_out"]) > TOL_LAYER[dt]
            print("fp8 layer", hidden, split, "err vs fp8 oracle", err, "rms", rms_rel_err(f64(xd), ref["x_out"]),
                  "vs exact", orc.max_rel_err(f64(xd), exact["x_out"]))


@pytest.mark.parametrize("name", ["30b_tp4_2k", "70b_tp8_4k"])
def test_full_size_fp8_projections_sampled_rows(name):
    wl = iso_inputs.WORKLOADS[name]
    dt = wl.dtype
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    rows = iso_inputs.sample_rows(wl.seq, wl.split, 48, seed=0)
    sh = shape_of(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn)
    ref = orc.layer_rows(h64(x, dt), oracle_weights(w, dt), sh, rows, fp8=True)
    with make_ctx(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, dt, wl.seq) as ctx:
        w_dev = ctx.add_fp8_weights(iso.upload_weights(w, dt))
        ctx.set_flags(iso.ISO_FLAG_FP8_GEMM)
        for split in (0, wl.split):
            xd = dev(x, dt)
            kc = iso.DeviceArray((wl.seq, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
            vc = iso.DeviceArray((wl.seq, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
            ctx.layer_prefill(w_dev, xd, kc, vc, wl.seq, split, iso.ISO_COMM_D2H)
            ctx.sync()
            err = orc.max_rel_err(f64(xd)[rows], ref["x_out"])
            print(name, "fp8 split", split, "err", err, "rms", rms_rel_err(f64(xd)[rows], ref["x_out"]))
            assert err <= TOL_LAYER_FP8, (split, err)
            assert rms_rel_err(f64(xd)[rows], ref["x_out"]) <= TOL_RMS_FP8
            assert orc.max_rel_err(f64(kc), ref["k_cache"]) <= TOL_LAYER_FP8
            assert rms_rel_err(f64(kc), ref["k_cache"]) <= TOL_RMS_FP8


def test_full_size_30b_tp4_2k_fp8_projection_from_the_devices_own_intermediate():
    """The layer bounds above are statistical (device and oracle quantise activations that differ by bf16 roundings),
    so a single wrong element could hide under them.  Here the oracle is fed the DEVICE's own bf16 intermediate: the
    norm output y of the full 30B TP=4 prompt is downloaded, the oracle quantises exactly those values and the
    weights (its quantiser is bit-identical to the device's), and every element of the device's FP8 QKV projection
    (2048 x 4992 x 6656, through the fused norm + quantiser as the layer runs it, and through the separate quantiser)
    must match the oracle's product at the single-step bound.  Then the same for o_proj fed the device's attention
    output."""
    wl = iso_inputs.WORKLOADS["30b_tp4_2k"]
    dt, T, H = wl.dtype, wl.seq, wl.hidden
    nqd = wl.n_q_heads * wl.head_dim
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    with make_ctx(H, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, dt, T) as ctx:
        s = ctx.stream0
        wd = ctx.add_fp8_weights(iso.upload_weights(w, dt))
        xd = dev(x, dt)
        y = iso.DeviceArray((T, H), dt)
        ctx.rmsnorm(xd, wd["g_attn"], y, T, s)
        a8, sa = iso.DeviceArray((T, H), "u8"), iso.DeviceArray((T,), "f32")
        ctx.rmsnorm_fp8(xd, None, wd["g_attn"], a8, sa, T, s)         # what the layer does under ISO_FLAG_FP8_GEMM
        qkv = iso.DeviceArray((T, wl.n_qkv), dt, fill_byte=NAN_BYTE)
        ctx.gemm_fp8(a8, sa, wd["w_qkv_f8"], wd["s_qkv"], qkv, T, wl.n_qkv, H, s)
        b8, sb = iso.DeviceArray((T, H), "u8"), iso.DeviceArray((T,), "f32")
        ctx.quantize_rows_fp8(y, T, H, b8, sb, s)                     # the separate quantiser on the stored y
        qkv2 = iso.DeviceArray((T, wl.n_qkv), dt, fill_byte=NAN_BYTE)
        ctx.gemm_fp8(b8, sb, wd["w_qkv_f8"], wd["s_qkv"], qkv2, T, wl.n_qkv, H, s)
        ctx.sync()
        ref = orc.linear_fp8(f64(y), h64(w["w_qkv"], dt))
        err = orc.max_rel_err(f64(qkv), ref)
        print("fp8 QKV from the device's own y: max_rel_err", err)
        assert err <= TOL_STEP[dt], err
        np.testing.assert_array_equal(qkv2.numpy(), qkv.numpy())
        # o_proj on the device's own attention output (bf16 layer run first to produce it through the library)
        kc = iso.DeviceArray((T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=0)
        vc = iso.DeviceArray((T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=0)
        ctx.rope_kv_write(qkv, kc, vc, T, 0, s)
        ctx.sync()
        q_only = dev(np.ascontiguousarray(qkv.numpy()[:, :nqd]), dt)
        att = iso.DeviceArray((T, nqd), dt)
        ctx.attn_chunk(q_only, kc, vc, att, T, 0, T, s)
        o8, so = iso.DeviceArray((T, nqd), "u8"), iso.DeviceArray((T,), "f32")
        ctx.quantize_rows_fp8(att, T, nqd, o8, so, s)
        pa = iso.DeviceArray((T, H), dt, fill_byte=NAN_BYTE)
        ctx.gemm_fp8(o8, so, wd["w_o_f8"], wd["s_o"], pa, T, H, nqd, s)
        ctx.sync()
        ref_o = orc.linear_fp8(f64(att), h64(w["w_o"], dt))
        err_o = orc.max_rel_err(f64(pa), ref_o)
        print("fp8 o_proj from the device's own attention output: max_rel_err", err_o)
        assert err_o <= TOL_STEP[dt], err_o


@pytest.mark.parametrize("hidden", [256, 6656, 8192])
@pytest.mark.parametrize("with_delta", [False, True])
def test_norm_with_fp8_tail_equals_norm_then_quantiser(hidden, with_delta):
    """The fused kernel must leave exactly the codes and scales that the row quantiser derives from the stored bf16
    norm output (and the same x + delta), and those codes are the oracle quantiser's for that output."""
    dt, T = "bf16", 37
    x = iso_inputs.make_hidden(T, hidden, seed=31, dtype=dt)
    x32 = iso_inputs.bf16_bits_to_f32(x)
    x32[4] = 0.0                                     # all-zero row: scale 1, codes 0
    x32[6] *= 1e-12
    x = iso_inputs.f32_to_bf16_bits(x32)
    delta = iso_inputs.randn((T, hidden), seed=32, dtype=dt, scale=0.5)
    if with_delta:
        d32 = iso_inputs.bf16_bits_to_f32(delta)
        d32[4] = 0.0
        delta = iso_inputs.f32_to_bf16_bits(d32)
    g = iso_inputs.randn((hidden,), seed=33, dtype=dt)
    with make_ctx(hidden, 2, 1, 128, 256, dt, 64) as ctx:
        gd = dev(g, dt)
        # separate kernels
        x_a, y = dev(x, dt), iso.DeviceArray((T, hidden), dt, fill_byte=NAN_BYTE)
        if with_delta:
            ctx.residual_rmsnorm(x_a, dev(delta, dt), gd, y, T, ctx.stream0)
        else:
            ctx.rmsnorm(x_a, gd, y, T, ctx.stream0)
        q_a, s_a = iso.DeviceArray((T, hidden), "u8", fill_byte=0x7F), iso.DeviceArray((T,), "f32")
        ctx.quantize_rows_fp8(y, T, hidden, q_a, s_a, ctx.stream0)
        # fused
        x_b = dev(x, dt)
        q_b, s_b = iso.DeviceArray((T, hidden), "u8", fill_byte=0x7F), iso.DeviceArray((T,), "f32")
        ctx.rmsnorm_fp8(x_b, dev(delta, dt) if with_delta else None, gd, q_b, s_b, T, ctx.stream0)
        ctx.sync()
        np.testing.assert_array_equal(q_b.numpy(), q_a.numpy())
        np.testing.assert_array_equal(s_b.numpy(), s_a.numpy())
        np.testing.assert_array_equal(x_b.numpy(), x_a.numpy())
        want_v, want_s = orc.quantize_rows_fp8(f64(y))
        np.testing.assert_array_equal(orc.fp8_e4m3_decode(q_b.numpy()), want_v)
        np.testing.assert_array_equal(s_b.numpy().astype(np.float64), want_s)


def test_norm_with_fp8_tail_rejects_wide_rows_and_fp32():
    with make_ctx(8320, 2, 1, 128, 256, "bf16", 16) as ctx:
        x = iso.DeviceArray((4, 8320), "bf16", fill_byte=0)
        q, s = iso.DeviceArray((4, 8320), "u8"), iso.DeviceArray((4,), "f32")
        g = iso.DeviceArray((8320,), "bf16", fill_byte=0)
        with pytest.raises(iso.IsoError) as ei:
            ctx.rmsnorm_fp8(x, None, g, q, s, 4, ctx.stream0)
        assert ei.value.code == iso.ISO_ERR_SHAPE
    with make_ctx(256, 4, 4, 64, 64, "f32", 16) as ctx:
        x = iso.DeviceArray((4, 256), "f32", fill_byte=0)
        q, s = iso.DeviceArray((4, 256), "u8"), iso.DeviceArray((4,), "f32")
        g = iso.DeviceArray((256,), "f32", fill_byte=0)
        with pytest.raises(iso.IsoError) as ei:
            ctx.rmsnorm_fp8(x, None, g, q, s, 4, ctx.stream0)
        assert ei.value.code == iso.ISO_ERR_DTYPE


def test_two_layer_stack_with_fp8_projections():
    """Layer 2's first norm closes layer 1 (x + attention partial + MLP partial): that variant of the fused norm +
    quantiser only runs inside a stack."""
    hidden, nq, nkv, d, ffn, T, dt = 512, 4, 1, 128, 768, 300, "bf16"
    layers = [iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=40 + l, dtype=dt) for l in range(2)]
    x = iso_inputs.make_hidden(T, hidden, seed=6, dtype=dt)
    sh = shape_of(hidden, nq, nkv, d, ffn)
    ref = h64(x, dt)
    for w in layers:
        ref = orc.layer_unsplit(ref, oracle_weights(w, dt), sh, fp8=True)["x_out"]
    with make_ctx(hidden, nq, nkv, d, ffn, dt, 320) as ctx:
        layers_dev = [ctx.add_fp8_weights(iso.upload_weights(w, dt)) for w in layers]
        ctx.set_flags(iso.ISO_FLAG_FP8_GEMM)
        outs = []
        for split in (0, 130):
            xd = dev(x, dt)
            kcs = iso.DeviceArray((2, 320, nkv, d), dt, fill_byte=NAN_BYTE)
            vcs = iso.DeviceArray((2, 320, nkv, d), dt, fill_byte=NAN_BYTE)
            ctx.stack_prefill(layers_dev, xd, kcs, vcs, T, split, iso.ISO_COMM_D2H)
            ctx.sync()
            err, rms = orc.max_rel_err(f64(xd), ref), rms_rel_err(f64(xd), ref)
            print("fp8 stack split", split, "err", err, "rms", rms)
            assert err <= 2 * TOL_LAYER_FP8 and rms <= 2 * TOL_RMS_FP8
            outs.append(xd.numpy())
