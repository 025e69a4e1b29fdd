"""GPU parity at depth and length: the 80-layer stack at its stated depth, the long prompts of Table 1 as whole
layers, a control that shows what the NaN-poisoned caches of the ordering tests would catch, and the error path of the
stream-K status word.

Tolerances as in test_gpu_parity.py: 2e-2 per bf16 layer (max |got - ref| / max(|ref|, rms(ref))), each layer checked
from the GPU's own input to that layer so that the bound is per layer and not compounded.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import paper_2409_11155_amd as iso      # first: binds libiso to the HIP runtime it was built against
import iso_inputs
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

TOL_LAYER = 2e-2
NAN_BYTE = 0xFF


def h64(a, dt="bf16"):
    return iso_inputs.to_f64(a, dt)


def dev(a, dt="bf16"):
    return iso.DeviceArray.from_numpy(a, dt)


def oracle_weights(w, dt="bf16"):
    return {k: h64(v, dt) for k, v in w.items()}


def shape_of(wl):
    return orc.LayerShape(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.rms_eps, wl.rope_base)


def make_ctx(wl, max_seq=None):
    return iso.Context(iso.make_cfg(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.dtype,
                                    max_seq or wl.seq))


# ------------------------------------------------------------------------------ the stack at its depth

def test_80_layer_stack_layers_0_1_39_79_each_from_the_gpus_own_input():
    """Section 2.2 (stacked transformer blocks): the 70B TP=8 stack at 80 layers, 16k prompt cut 8192/8192, one
    seed per layer, KV cache of every layer kept, both chunks on their streams from the first layer to the last, the
    copy stand-in at both communication points.  Layers 0, 1, 39 and 79 are checked against the oracle, each fed the
    GPU's own input to that layer (the output of the stack's first l layers; a stack of l layers and the first l
    layers of a deeper stack run the same launches, and repeated runs are bit-identical), on sampled rows plus every
    K/V row the 80-layer run left in that layer's cache."""
    wl = iso_inputs.WORKLOADS["70b_tp8_16k_stack"]
    dt, T, split, L = wl.dtype, wl.seq, wl.split, wl.n_layers
    assert L == 80
    check = [0, 1, 39, 79]

    def draw(l):
        return iso_inputs.make_layer(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, seed=1000 + l, dtype=dt)

    kept, layers_dev = {}, []
    with ThreadPoolExecutor(8) as ex:
        for l, w in enumerate(ex.map(draw, range(L))):
            layers_dev.append(iso.upload_weights(w, dt))
            if l in check:
                kept[l] = w
    x0 = iso_inputs.make_hidden(T, wl.hidden, seed=0, dtype=dt)
    rows = iso_inputs.sample_rows(T, split, 24, seed=2)
    sh = shape_of(wl)
    prefix = sorted({l for l in check} | {l + 1 for l in check})          # 0, 1, 2, 39, 40, 79, 80
    outs = {0: x0}
    caches = {}
    with make_ctx(wl) as ctx:
        kcs = iso.DeviceArray((L, T, wl.n_kv_heads, wl.head_dim), dt)
        vcs = iso.DeviceArray((L, T, wl.n_kv_heads, wl.head_dim), dt)
        for n in prefix:
            if n == 0:
                continue
            xd = dev(x0, dt)
            kcs.fill(NAN_BYTE)
            vcs.fill(NAN_BYTE)
            ctx.stack_prefill(layers_dev[:n], xd, kcs, vcs, T, split, iso.ISO_COMM_D2H, iso.ISO_SCHED_OVERLAP)
            ctx.sync()
            outs[n] = xd.numpy()
            xd.free()
            if n == L:
                k_all, v_all = kcs.numpy(), vcs.numpy()
                caches = {l: (k_all[l], v_all[l]) for l in check}
                del k_all, v_all
    final = iso_inputs.bf16_bits_to_f32(outs[L])
    assert np.isfinite(final).all(), "the 80-layer output holds a non-finite value"
    errs = {}
    for l in check:
        ref = orc.layer_rows(h64(outs[l], dt), oracle_weights(kept[l], dt), sh, rows)
        err = orc.max_rel_err(h64(outs[l + 1], dt)[rows], ref["x_out"])
        ek = orc.max_rel_err(h64(caches[l][0], dt), ref["k_cache"])
        ev = orc.max_rel_err(h64(caches[l][1], dt), ref["v_cache"])
        errs[l] = (err, ek, ev)
        assert err <= TOL_LAYER and ek <= TOL_LAYER and ev <= TOL_LAYER, (l, err, ek, ev)
    rms = {n: float(np.sqrt(np.mean(iso_inputs.bf16_bits_to_f32(outs[n]).astype(np.float64) ** 2))) for n in outs}
    print("80-layer stack: per-layer max_rel_err (x_out, k, v):", errs, "rms of the residual stream:", rms)


# ------------------------------------------------------------------------------ long prompts as whole layers

def _long_prompt_layer(name, n_rows):
    wl = iso_inputs.WORKLOADS[name]
    dt, T, split = wl.dtype, wl.seq, wl.split
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    rows = iso_inputs.sample_rows(T, split, n_rows, seed=0)
    ref = orc.layer_rows(h64(x, dt), oracle_weights(w, dt), shape_of(wl), rows)
    with make_ctx(wl) as ctx:
        xd = dev(x, dt)
        kc = iso.DeviceArray((T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
        vc = iso.DeviceArray((T, wl.n_kv_heads, wl.head_dim), dt, fill_byte=NAN_BYTE)
        ctx.layer_prefill(iso.upload_weights(w, dt), xd, kc, vc, T, split, iso.ISO_COMM_D2H, iso.ISO_SCHED_OVERLAP)
        ctx.sync()
        got = xd.numpy()[rows]
        ek = orc.max_rel_err(h64(kc.numpy(), dt), ref["k_cache"])
        ev = orc.max_rel_err(h64(vc.numpy(), dt), ref["v_cache"])
    err = orc.max_rel_err(h64(got, dt), ref["x_out"])
    print(name, "ISO layer, sampled rows: max_rel_err", err, "k", ek, "v", ev)
    assert err <= TOL_LAYER and ek <= TOL_LAYER and ev <= TOL_LAYER, (name, err, ek, ev)


def test_full_size_70b_tp8_64k_layer_sampled_rows():
    """Table 1's 64k column at the 70B TP=8 shard: the whole ISO layer (projections at M = 37888 / 27648)."""
    _long_prompt_layer("70b_tp8_64k", 32)


def test_full_size_70b_tp8_128k_layer_sampled_rows():
    """Table 1's 128k column: the whole ISO layer (projections at M = 77824 / 53248, attention over 131072 keys)."""
    _long_prompt_layer("70b_tp8_128k", 32)


# ------------------------------------------------------------------------------ what the poisoned caches catch

@pytest.mark.parametrize("dt,d,flags", [("bf16", 128, 0), ("bf16", 128, iso.ISO_FLAG_ATTN_STAGED), ("bf16", 64, 0),
                                        ("f32", 64, 0)])
def test_attention_over_unwritten_cache_rows_gives_nan(dt, d, flags):
    """Control for the ordering tests (Section 3.1: chunk 1 reads what chunk 0 wrote): they start from NaN-filled
    caches and require a NaN-free result.  Here the rows [0, q_offset) of the caches are left as the poison, as if
    chunk 0 had not written them yet, and only the chunk's own rows are valid: every output row sees key 0, so every
    output element must be NaN.  A kernel that skipped, clamped or masked such rows would make those tests vacuous."""
    Tc, q_offset, nq, nkv = 200, 136, 4, 2
    kv_len = q_offset + Tc
    q, k, v = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=5, dtype=dt)
    nan_bits = np.uint16(0xFFFF) if dt == "bf16" else np.float32(np.nan)
    k[:q_offset] = nan_bits
    v[:q_offset] = nan_bits
    with iso.Context(iso.make_cfg(256, nq, nkv, d, 64, dt, kv_len)) as ctx:
        ctx.set_flags(flags)
        out = iso.DeviceArray((Tc, nq * d), dt, fill_byte=0)
        ctx.attn_chunk(dev(q, dt), dev(k, dt), dev(v, dt), out, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        got = h64(out.numpy(), dt)
        assert np.isnan(got).all(), f"{np.isnan(got).mean():.3f} of the outputs are NaN, expected all"
        # and with the rows written the same call is NaN-free and matches the oracle
        q2, k2, v2 = iso_inputs.make_qkv_cache(Tc, kv_len, nq, nkv, d, seed=5, dtype=dt)
        ctx.attn_chunk(dev(q2, dt), dev(k2, dt), dev(v2, dt), out, Tc, q_offset, kv_len, ctx.stream0)
        ctx.sync()
        got = h64(out.numpy(), dt)
        ref = orc.attention_chunk(h64(q2, dt), h64(k2, dt), h64(v2, dt), q_offset, kv_len).reshape(Tc, nq * d)
        assert not np.isnan(got).any()
        assert orc.max_rel_err(got, ref) <= (2e-5 if dt == "f32" else 3e-2)


def test_layer_with_chunk_0_rows_missing_from_the_cache_is_caught_by_the_poison():
    """The same control one level up: chunk 1 of a layer run on its own (rows [split, T) as a prompt placed at
    q_offset = split through the step entry points) over caches whose first `split` rows are still poison gives NaN
    attention output, while the library's ISO schedule over the same poisoned caches does not."""
    hidden, nq, nkv, d, ffn, T, split, dt = 512, 4, 1, 128, 512, 384, 160, "bf16"
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=41, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=41, dtype=dt)
    wd = iso.upload_weights(w, dt)
    nqkv = (nq + 2 * nkv) * d
    with iso.Context(iso.make_cfg(hidden, nq, nkv, d, ffn, dt, T)) as ctx:
        kc = iso.DeviceArray((T, nkv, d), dt, fill_byte=NAN_BYTE)
        vc = iso.DeviceArray((T, nkv, d), dt, fill_byte=NAN_BYTE)
        n1 = T - split
        x1 = dev(x[split:], dt)
        y = iso.DeviceArray((n1, hidden), dt)
        qkv = iso.DeviceArray((n1, nqkv), dt)
        qonly = iso.DeviceArray((n1, nq * d), dt)
        att = iso.DeviceArray((n1, nq * d), dt, fill_byte=0)
        s = ctx.stream0
        ctx.rmsnorm(x1, wd["g_attn"], y, n1, s)
        ctx.gemm_rowpar(y, wd["w_qkv"], qkv, n1, nqkv, hidden, s)
        ctx.rope_kv_write(qkv, kc, vc, n1, split, s)
        ctx.sync()
        qonly.upload(np.ascontiguousarray(qkv.numpy()[:, : nq * d]))
        ctx.attn_chunk(qonly, kc, vc, att, n1, split, T, s)     # chunk 0 never wrote rows [0, split)
        ctx.sync()
        assert np.isnan(h64(att.numpy(), dt)).all()
        # the library's own schedule over equally poisoned caches: chunk 0 writes first, nothing is NaN
        xd = dev(x, dt)
        kc.fill(NAN_BYTE)
        vc.fill(NAN_BYTE)
        ctx.layer_prefill(wd, xd, kc, vc, T, split, iso.ISO_COMM_D2H, iso.ISO_SCHED_OVERLAP)
        ctx.sync()
        got = h64(xd.numpy(), dt)
        assert not np.isnan(got).any()
        ref = orc.layer_unsplit(h64(x, dt), oracle_weights(w, dt), orc.LayerShape(hidden, nq, nkv, d, ffn))
        assert orc.max_rel_err(got, ref["x_out"]) <= TOL_LAYER


# ------------------------------------------------------------------------------ stream-K status word

def test_stream_k_status_word_is_sticky_until_sync_reports_it():
    """A stream-K wait that ran out is reported through a pinned word.  No kernel is made to time out: the test
    writes the word itself and expects every compute entry point to refuse work, iso_sync to report the error once
    and clear it, and iso_destroy to report it if it is still set."""
    hidden, nq, nkv, d, ffn, T, dt = 256, 2, 1, 128, 256, 128, "bf16"
    w = iso.upload_weights(iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=1, dtype=dt), dt)
    x = iso_inputs.make_hidden(T, hidden, seed=1, dtype=dt)
    cfg = iso.make_cfg(hidden, nq, nkv, d, ffn, dt, T)
    ctx = iso.Context(cfg)
    xd = dev(x, dt)
    kc = iso.DeviceArray((T, nkv, d), dt, fill_byte=0)
    vc = iso.DeviceArray((T, nkv, d), dt, fill_byte=0)
    word = ctx.streamk_status_word()
    assert word is not None and word[0] == 0
    ctx.layer_prefill(w, xd, kc, vc, T, 64)
    ctx.sync()
    before = xd.numpy().copy()
    word[0] = 1
    for call in (lambda: ctx.layer_prefill(w, xd, kc, vc, T, 64),
                 lambda: ctx.stack_prefill([w], xd, kc, vc, T, 64),
                 lambda: ctx.stack_prefill_chunks([w], xd, kc, vc, T, [32, 64]),
                 lambda: ctx.gemm_rowpar(xd, w["w_qkv"], xd, 8, 8, hidden, ctx.stream0),
                 lambda: ctx.attn_chunk(xd, kc, vc, xd, 1, 0, 1, ctx.stream0)):
        with pytest.raises(iso.IsoError) as ei:
            call()
        assert ei.value.code == iso.ISO_ERR_HIP
    with pytest.raises(iso.IsoError) as ei:
        ctx.sync()
    assert ei.value.code == iso.ISO_ERR_HIP and "stream-K" in str(ei.value)
    np.testing.assert_array_equal(xd.numpy(), before)       # nothing was enqueued while the word was set
    assert word[0] == 0
    ctx.sync()                                               # reported once, then clear
    ctx.layer_prefill(w, xd, kc, vc, T, 64)
    ctx.sync()
    word[0] = 1
    assert ctx.close() == iso.ISO_ERR_HIP
    # an fp32 context has no stream-K kernel and no word
    with iso.Context(iso.make_cfg(256, 4, 4, 64, 64, "f32", 64)) as c32:
        assert c32.streamk_status_word() is None
