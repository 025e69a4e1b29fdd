"""Pins for the CPU oracle: everything here checks oracle/ against something that is
not the oracle -- closed forms, scalar brute force on tiny inputs, library routines on
special cases, and the invariants the paper states (Section 3.1: chunking over the KV
cache introduces no error, for any split point).  No GPU is used.
"""
import json
import math
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

import iso_inputs
from oracle import iso_oracle as orc

RNG = np.random.default_rng(1234)


# ------------------------------------------------------------------ linear

def test_linear_matches_scalar_loops_and_is_not_transposed():
    a = RNG.standard_normal((3, 5))
    w = RNG.standard_normal((4, 5))           # [N, K]: non-square, so a transposed operand cannot pass
    c = orc.linear(a, w)
    assert c.shape == (3, 4)
    for t in range(3):
        for n in range(4):
            acc = 0.0
            for k in range(5):
                acc += a[t, k] * w[n, k]
            assert c[t, n] == pytest.approx(acc, rel=1e-14, abs=1e-14)


def test_linear_onehot_selects_weight_column_and_identity_copies():
    w = RNG.standard_normal((6, 4))
    e2 = np.zeros((1, 4)); e2[0, 2] = 1.0
    np.testing.assert_array_equal(orc.linear(e2, w)[0], w[:, 2])
    a = RNG.standard_normal((5, 4))
    np.testing.assert_array_equal(orc.linear(a, np.eye(4)), a)


# ------------------------------------------------------------------ rmsnorm

def test_rmsnorm_hand_value():
    # x = (3, 4): mean square 12.5, eps 0.5 -> divide by sqrt(13)
    y = orc.rmsnorm(np.array([[3.0, 4.0]]), np.array([2.0, -1.0]), 0.5)
    np.testing.assert_allclose(y, [[6.0 / math.sqrt(13.0), -4.0 / math.sqrt(13.0)]], rtol=1e-15)


def test_rmsnorm_unit_mean_square_and_scale_invariance():
    x = RNG.standard_normal((7, 64)) * 3.0
    g = np.ones(64)
    eps = 1e-6
    y = orc.rmsnorm(x, g, eps)
    ms = np.mean(x * x, axis=1)
    np.testing.assert_allclose(np.mean(y * y, axis=1), ms / (ms + eps), rtol=1e-13)
    np.testing.assert_allclose(orc.rmsnorm(1e3 * x, g, 0.0), orc.rmsnorm(x, g, 0.0), rtol=1e-13)
    # eps sits inside the square root, next to the mean (not added to the root)
    y0 = orc.rmsnorm(np.zeros((1, 4)) + 1e-9, np.ones(4), 1.0)
    np.testing.assert_allclose(y0, 1e-9 / math.sqrt(1.0 + 1e-18), rtol=1e-12)


# ------------------------------------------------------------------ rope

def test_rope_d2_is_a_plane_rotation_by_the_position():
    a = np.array([[[1.0, 0.0]], [[0.0, 1.0]], [[2.0, -3.0]]])       # [t=3, heads=1, d=2]
    pos = np.array([0, 1, 5])
    out = orc.rope(a, pos, 10000.0)                                  # theta_0 = 1 for d = 2
    np.testing.assert_allclose(out[0, 0], [1.0, 0.0], atol=0)        # position 0 is the identity
    np.testing.assert_allclose(out[1, 0], [-math.sin(1.0), math.cos(1.0)], rtol=1e-15)
    c, s = math.cos(5.0), math.sin(5.0)
    np.testing.assert_allclose(out[2, 0], [2 * c + 3 * s, -3 * c + 2 * s], rtol=1e-14)


def test_rope_pairs_are_i_and_i_plus_half_with_geometric_frequencies():
    # d = 4, base 10000: theta_0 = 1, theta_1 = 10000^(-2/4) = 0.01.  At position 100 the pair
    # (1, 3) turns by exactly 1 rad and the pair (0, 2) by 100 rad.
    a = np.zeros((1, 1, 4)); a[0, 0, 1] = 1.0
    out = orc.rope(a, np.array([100]), 10000.0)[0, 0]
    np.testing.assert_allclose(out, [0.0, math.cos(1.0), 0.0, math.sin(1.0)], atol=1e-13)
    a = np.zeros((1, 1, 4)); a[0, 0, 2] = 1.0
    out = orc.rope(a, np.array([100]), 10000.0)[0, 0]
    np.testing.assert_allclose(out, [-math.sin(100.0), 0.0, math.cos(100.0), 0.0], atol=1e-13)


def test_rope_preserves_norm_and_scores_depend_on_relative_position_only():
    d = 16
    q = RNG.standard_normal((1, 1, d))
    k = RNG.standard_normal((1, 1, d))
    def score(m, n):
        return float(np.sum(orc.rope(q, np.array([m]), 10000.0) * orc.rope(k, np.array([n]), 10000.0)))
    assert score(17, 5) == pytest.approx(score(112, 100), rel=1e-12)
    assert score(17, 5) != pytest.approx(score(5, 17), rel=1e-6)      # direction matters
    r = orc.rope(q, np.array([977]), 10000.0)
    assert np.linalg.norm(r) == pytest.approx(np.linalg.norm(q), rel=1e-14)


# ------------------------------------------------------------------ silu / swiglu

def test_silu_values_and_identities():
    assert orc.silu(0.0) == 0.0
    assert float(orc.silu(1.0)) == pytest.approx(1.0 / (1.0 + math.exp(-1.0)), rel=1e-15)
    assert float(orc.silu(-1.0)) == pytest.approx(-1.0 / (1.0 + math.e), rel=1e-15)
    z = RNG.standard_normal(50) * 4
    np.testing.assert_allclose(orc.silu(-z), orc.silu(z) - z, atol=1e-14)
    assert float(orc.silu(40.0)) == pytest.approx(40.0, rel=1e-15)


def test_swiglu_gate_is_first_half_up_is_second_half():
    gu = np.array([[1.0, -2.0, 10.0, 100.0]])        # gate = (1, -2), up = (10, 100)
    out = orc.swiglu(gu)
    np.testing.assert_allclose(out, [[10.0 / (1 + math.exp(-1.0)), -200.0 / (1 + math.exp(2.0))]], rtol=1e-15)


# ------------------------------------------------------------------ attention

def brute_force_attention(q, k, v, q_offset, kv_len):
    """Masked [Tc, kv] score matrix + library softmax, written independently of the oracle."""
    Tc, nq, d = q.shape
    nkv = k.shape[1]
    out = np.zeros((Tc, nq, d))
    for h in range(nq):
        g = h * nkv // nq
        s = np.einsum("id,jd->ij", q[:, h], k[:kv_len, g]) / math.sqrt(d)
        i = np.arange(Tc)[:, None]
        j = np.arange(kv_len)[None, :]
        s = np.where(j <= q_offset + i, s, -np.inf)
        out[:, h] = sp_softmax(s, axis=1) @ v[:kv_len, g]
    return out


@pytest.mark.parametrize("nq,nkv", [(1, 1), (2, 1), (4, 2), (8, 1), (4, 4)])
def test_attention_chunk_equals_brute_force_for_every_chunk_placement(nq, nkv):
    T, d = 10, 8
    q_all = RNG.standard_normal((T, nq, d))
    k = RNG.standard_normal((T, nkv, d))
    v = RNG.standard_normal((T, nkv, d))
    for q_offset in range(T):
        for Tc in range(1, T - q_offset + 1):
            q = q_all[q_offset:q_offset + Tc]
            got = orc.attention_chunk(q, k, v, q_offset, q_offset + Tc)
            ref = brute_force_attention(q, k, v, q_offset, q_offset + Tc)
            np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_attention_chunk_kv_len_truncates_visible_keys():
    T, d = 9, 4
    q = RNG.standard_normal((4, 2, d)); k = RNG.standard_normal((T, 1, d)); v = RNG.standard_normal((T, 1, d))
    got = orc.attention_chunk(q, k, v, q_offset=5, kv_len=7)       # rows 5..8 but only keys 0..6 exist
    ref = brute_force_attention(q, k, v, 5, 7)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-13)


def test_attention_full_equals_brute_force_and_chunk_from_zero():
    T, d = 13, 8
    q = RNG.standard_normal((T, 4, d)); k = RNG.standard_normal((T, 2, d)); v = RNG.standard_normal((T, 2, d))
    ref = brute_force_attention(q, k, v, 0, T)
    np.testing.assert_allclose(orc.attention_full(q, k, v), ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.attention_chunk(q, k, v, 0, T), ref, rtol=1e-12, atol=1e-13)


def test_attention_degenerate_cases():
    T, d = 11, 8
    q = RNG.standard_normal((T, 2, d)); k = RNG.standard_normal((T, 1, d)); v = RNG.standard_normal((T, 1, d))
    for fn in (lambda q_, k_, v_: orc.attention_full(q_, k_, v_),
               lambda q_, k_, v_: orc.attention_chunk(q_, k_, v_, 0, T)):
        out = fn(q, k, v)
        # first token sees only itself
        np.testing.assert_allclose(out[0, 0], v[0, 0], rtol=1e-14)
        np.testing.assert_allclose(out[0, 1], v[0, 0], rtol=1e-14)
        # identical keys -> uniform weights -> running mean of v
        k_same = np.broadcast_to(k[:1], k.shape)
        out = fn(q, k_same, v)
        for t in range(T):
            np.testing.assert_allclose(out[t, 0], v[:t + 1, 0].mean(axis=0), rtol=1e-12, atol=1e-14)
        # constant v -> constant output (weights sum to one)
        out = fn(q, k, np.full_like(v, 2.5))
        np.testing.assert_allclose(out, 2.5, rtol=1e-13)
        # adding one vector to every key shifts all scores of a row equally: no change
        out = fn(q, k + RNG.standard_normal((1, 1, d)), v)
        np.testing.assert_allclose(out, fn(q, k, v), rtol=1e-9, atol=1e-11)


def test_attention_uses_scale_one_over_sqrt_d():
    # one query, two keys with scores ln(3)*sqrt(d) and 0 before scaling -> weights 3/4, 1/4
    d = 4
    q = np.zeros((1, 1, d)); q[0, 0, 0] = 1.0
    k = np.zeros((2, 1, d)); k[1, 0, 0] = math.log(3.0) * math.sqrt(d)
    v = np.zeros((2, 1, d)); v[0, 0, 0] = 1.0; v[1, 0, 1] = 1.0
    out = orc.attention_chunk(q, k, v, q_offset=1, kv_len=2)
    np.testing.assert_allclose(out[0, 0, :2], [0.25, 0.75], rtol=1e-14)


def test_gqa_head_mapping_is_contiguous_groups():
    # 4 query heads over 2 kv heads: heads 0,1 read kv head 0; heads 2,3 read kv head 1
    T, d = 3, 4
    q = RNG.standard_normal((T, 4, d)); k = RNG.standard_normal((T, 2, d))
    v = np.zeros((T, 2, d)); v[:, 0, :] = 1.0; v[:, 1, :] = -1.0
    out = orc.attention_full(q, k, v)
    np.testing.assert_allclose(out[:, :2], 1.0, rtol=1e-14)
    np.testing.assert_allclose(out[:, 2:], -1.0, rtol=1e-14)
    out = orc.attention_chunk(q, k, v, 0, T)
    np.testing.assert_allclose(out[:, :2], 1.0, rtol=1e-14)
    np.testing.assert_allclose(out[:, 2:], -1.0, rtol=1e-14)


# ------------------------------------------------------------------ whole layer

def _np_weights(w, dtype="f32"):
    return {k: iso_inputs.to_f64(v, dtype) for k, v in w.items()}


def _tiny():
    wl = iso_inputs.WORKLOADS["tiny_f32"]
    x, w = iso_inputs.make_workload_inputs(wl, seed=0)
    sh = orc.LayerShape(wl.hidden, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.ffn, wl.rms_eps, wl.rope_base)
    return wl, iso_inputs.to_f64(x, wl.dtype), _np_weights(w, wl.dtype), sh


def test_two_token_layer_closed_form():
    """H = d = 2, one head, ffn 1, identity projections: every intermediate has a closed form.
    token 0 = (1,1), token 1 = (1,-1), eps = 0.  RoPE with d = 2 rotates by `position` radians.
    q1 = k1 = R(1)(1,-1) = (cos1 + sin1, sin1 - cos1);  scores of row 1: sqrt2*sin1 and sqrt2,
    so o1 = (1, tanh(sqrt2 (sin1 - 1)/2)); o0 = v0 = (1,1)."""
    sh = orc.LayerShape(hidden=2, n_q_heads=1, n_kv_heads=1, head_dim=2, ffn=1, rms_eps=0.0, rope_base=10000.0)
    eye = np.eye(2)
    w = {"w_qkv": np.vstack([eye, eye, eye]), "w_o": eye,
         "w_gate_up": np.array([[1.0, 0.0], [0.0, 1.0]]),           # gate = y2[0], up = y2[1]
         "w_down": np.array([[1.0], [0.0]]),                        # MLP output lands in column 0
         "g_attn": np.ones(2), "g_mlp": np.ones(2)}
    x = np.array([[1.0, 1.0], [1.0, -1.0]])
    c = -1.0 + math.tanh(math.sqrt(2.0) * (math.sin(1.0) - 1.0) / 2.0)
    x1 = np.array([[2.0, 2.0], [2.0, c]])
    ms1 = (4.0 + c * c) / 2.0
    gate1, up1 = 2.0 / math.sqrt(ms1), c / math.sqrt(ms1)
    want = np.array([[2.0 + 1.0 / (1.0 + math.exp(-1.0)), 2.0],
                     [2.0 + gate1 / (1.0 + math.exp(-gate1)) * up1, c]])
    for res in (orc.layer_unsplit(x, w, sh), orc.layer_iso(x, w, sh, 1), orc.layer_rows(x, w, sh, [0, 1])):
        np.testing.assert_allclose(res["x1"], x1, rtol=1e-14)
        np.testing.assert_allclose(res["x_out"], want, rtol=1e-14)
        np.testing.assert_allclose(res["k_cache"][1, 0], [math.cos(1) + math.sin(1), math.sin(1) - math.cos(1)],
                                   rtol=1e-14)
        np.testing.assert_allclose(res["v_cache"][1, 0], [1.0, -1.0], rtol=1e-14)


def scalar_layer(x, w, sh):
    """The layer in pure-Python scalar loops (only `math`), for tiny shapes."""
    T, H = len(x), sh.hidden
    nq, nkv, d, F = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn
    half = d // 2

    def norm(row, g):
        ms = sum(val * val for val in row) / H
        return [row[i] / math.sqrt(ms + sh.rms_eps) * g[i] for i in range(H)]

    def matvec(wm, vec):
        return [sum(wm[n][k_] * vec[k_] for k_ in range(len(vec))) for n in range(len(wm))]

    def rot(vec, p):
        out = list(vec)
        for i in range(half):
            th = p * sh.rope_base ** (-2.0 * i / d)
            out[i] = vec[i] * math.cos(th) - vec[i + half] * math.sin(th)
            out[i + half] = vec[i + half] * math.cos(th) + vec[i] * math.sin(th)
        return out

    qs, ks, vs = [], [], []
    for t in range(T):
        qkv = matvec(w["w_qkv"], norm(x[t], w["g_attn"]))
        qs.append([rot(qkv[h * d:(h + 1) * d], t) for h in range(nq)])
        ks.append([rot(qkv[(nq + g) * d:(nq + g + 1) * d], t) for g in range(nkv)])
        vs.append([qkv[(nq + nkv + g) * d:(nq + nkv + g + 1) * d] for g in range(nkv)])
    out = []
    for t in range(T):
        o = []
        for h in range(nq):
            g = h // (nq // nkv)
            sc = [sum(qs[t][h][i] * ks[j][g][i] for i in range(d)) / math.sqrt(d) for j in range(t + 1)]
            m = max(sc)
            e = [math.exp(s_ - m) for s_ in sc]
            z = sum(e)
            o += [sum(e[j] / z * vs[j][g][i] for j in range(t + 1)) for i in range(d)]
        pa = matvec(w["w_o"], o)
        x1 = [x[t][i] + pa[i] for i in range(H)]
        gu = matvec(w["w_gate_up"], norm(x1, w["g_mlp"]))
        a = [gu[f] / (1.0 + math.exp(-gu[f])) * gu[F + f] for f in range(F)]
        pm = matvec(w["w_down"], a)
        out.append([x1[i] + pm[i] for i in range(H)])
    return np.array(out)


@pytest.mark.parametrize("nq,nkv", [(2, 1), (2, 2), (4, 2)])
def test_layer_equals_scalar_brute_force_on_tiny_shapes(nq, nkv):
    sh = orc.LayerShape(hidden=6, n_q_heads=nq, n_kv_heads=nkv, head_dim=4, ffn=5, rms_eps=1e-6, rope_base=10000.0)
    w = _np_weights(iso_inputs.make_layer(6, nq, nkv, 4, 5, seed=3, dtype="f32"))
    x = iso_inputs.to_f64(iso_inputs.make_hidden(5, 6, seed=3, dtype="f32"), "f32")
    want = scalar_layer(x.tolist(), {k: v.tolist() for k, v in w.items()}, sh)
    np.testing.assert_allclose(orc.layer_unsplit(x, w, sh)["x_out"], want, rtol=1e-12, atol=1e-13)
    for s in range(1, 5):
        np.testing.assert_allclose(orc.layer_iso(x, w, sh, s)["x_out"], want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(orc.layer_rows(x, w, sh, [4, 0, 2])["x_out"], want[[4, 0, 2]], rtol=1e-12, atol=1e-13)


def test_zero_output_projections_make_the_layer_an_identity():
    wl, x, w, sh = _tiny()
    w = dict(w, w_o=np.zeros_like(w["w_o"]), w_down=np.zeros_like(w["w_down"]))
    np.testing.assert_array_equal(orc.layer_unsplit(x, w, sh)["x_out"], x)
    np.testing.assert_array_equal(orc.layer_iso(x, w, sh, 50)["x_out"], x)


def test_split_invariance_for_every_split_point():
    """Section 3.1: a chunk that reads the KV cache of the earlier chunk reproduces the
    unsplit prefill.  Checked for all 127 split points of the small workload."""
    wl, x, w, sh = _tiny()
    ref = orc.layer_unsplit(x, w, sh)
    for s in range(1, wl.seq):
        got = orc.layer_iso(x, w, sh, s)
        assert orc.max_rel_err(got["x_out"], ref["x_out"]) < 1e-12, s
        assert orc.max_rel_err(got["k_cache"], ref["k_cache"]) < 1e-13, s
        assert orc.max_rel_err(got["v_cache"], ref["v_cache"]) < 1e-13, s


def test_split_invariance_for_finer_cuts():
    """Section 6: any finer segmentation of the prompt is still the same layer.  Random partitions into
    3..8 chunks, including one-token chunks, against the unsplit prefill."""
    wl, x, w, sh = _tiny()
    ref = orc.layer_unsplit(x, w, sh)
    gen = np.random.default_rng(5)
    cases = [[1, 2], [wl.seq - 2, wl.seq - 1], list(range(16, wl.seq, 16))]
    for n in range(3, 9):
        cases.append(sorted(int(c) for c in gen.choice(np.arange(1, wl.seq), size=n - 1, replace=False)))
    for cuts in cases:
        got = orc.layer_iso(x, w, sh, cuts)
        assert orc.max_rel_err(got["x_out"], ref["x_out"]) < 1e-12, cuts
        assert orc.max_rel_err(got["k_cache"], ref["k_cache"]) < 1e-13, cuts
    for bad in ([0], [wl.seq], [40, 40], [50, 30]):
        with pytest.raises(ValueError):
            orc.layer_iso(x, w, sh, bad)


def test_token_cost_and_balanced_cuts():
    """Section 6: cut by cost, not by length.  Pins: the hand-computed cost of one position; without an
    attention term the cuts are equal lengths; with it every chunk costs the same to within one token and
    the first chunk is the longest; the two-chunk cut solves the quadratic of the continuous cost."""
    sh = orc.LayerShape(hidden=8, n_q_heads=2, n_kv_heads=1, head_dim=4, ffn=16, rms_eps=1e-6, rope_base=1e4)
    # projections: qkv 2*8*(2+2)*4 = 256, o 2*8*8 = 128, gate/up/down 6*8*16 = 768 -> 1152; attention at
    # position 2 (3 keys): 4 * 2 * 4 * 3 = 96 flops, weighted by 2.5
    assert orc.token_cost(sh, 5, 2.5)[2] == 1152 + 2.5 * 96
    np.testing.assert_allclose(orc.balanced_cuts(sh, 120, 4, 0.0), [30, 60, 90], rtol=0, atol=1e-9)
    big = orc.LayerShape(hidden=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, ffn=2048, rms_eps=1e-6, rope_base=1e4)
    T, n = 4096, 4
    cost = orc.token_cost(big, T, 3.0)
    cuts = orc.balanced_cuts(big, T, n, 3.0)
    edges = np.concatenate([[0], np.round(cuts).astype(int), [T]])
    per_chunk = np.array([cost[a:b].sum() for a, b in zip(edges[:-1], edges[1:])])
    assert np.all(np.abs(per_chunk - cost.sum() / n) <= cost.max())
    lengths = np.diff(edges)
    assert np.all(np.diff(lengths) < 0)          # strictly shorter chunks towards the dear end
    # two chunks: proj * t + a * t * (t + 1) = total / 2 with a = 3 * 2 * nq * d
    proj, a = cost[0] - 3.0 * 4 * 8 * 128, 3.0 * 2 * 8 * 128
    t = orc.balanced_cuts(big, T, 2, 3.0)[0]
    assert abs(proj * t + a * t * (t + 1) - cost.sum() / 2) <= cost.max()


def test_causality_later_tokens_do_not_touch_earlier_rows():
    wl, x, w, sh = _tiny()
    p = 40
    x2 = x.copy()
    x2[p:] += RNG.standard_normal(x2[p:].shape)
    a = orc.layer_unsplit(x, w, sh)["x_out"]
    b = orc.layer_unsplit(x2, w, sh)["x_out"]
    np.testing.assert_allclose(a[:p], b[:p], rtol=1e-13, atol=1e-14)
    assert np.abs(a[p:] - b[p:]).max() > 1e-2
    a = orc.layer_iso(x, w, sh, 64)["x_out"]
    b = orc.layer_iso(x2, w, sh, 64)["x_out"]
    np.testing.assert_array_equal(a[:p], b[:p])


def test_chunk_one_uses_absolute_positions():
    """If chunk 1 restarted its positions at zero the split result would differ: make sure the
    invariance test above has teeth by checking that RoPE positions matter at this size."""
    wl, x, w, sh = _tiny()
    T = wl.seq
    y = orc.rmsnorm(x, w["g_attn"], sh.rms_eps)
    q, k, v = orc._split_qkv(orc.linear(y, w["w_qkv"]), sh)
    right = orc.rope(k[64:], np.arange(64, T), sh.rope_base)
    wrong = orc.rope(k[64:], np.arange(0, T - 64), sh.rope_base)
    assert np.abs(right - wrong).max() > 0.1
    np.testing.assert_allclose(orc.layer_iso(x, w, sh, 64)["k_cache"][64:], right, rtol=1e-13, atol=1e-14)


def test_layer_rows_equal_full_layer_rows():
    wl, x, w, sh = _tiny()
    rows = iso_inputs.sample_rows(wl.seq, wl.split, 16, seed=1)
    assert {0, 1, wl.split - 1, wl.split, wl.split + 1, wl.seq - 1} <= set(rows)
    full = orc.layer_unsplit(x, w, sh)
    part = orc.layer_rows(x, w, sh, rows)
    np.testing.assert_allclose(part["x_out"], full["x_out"][rows], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(part["k_cache"], full["k_cache"], rtol=1e-13, atol=1e-14)


def test_stored_oracle_values_still_reproduce():
    """tests/golden/tiny_f32_oracle.json is written by tests/golden/make_golden.py from oracle/
    alone; a silent change of the oracle's arithmetic or of the input recipe shows up here."""
    path = os.path.join(os.path.dirname(__file__), "golden", "tiny_f32_oracle.json")
    with open(path) as f:
        gold = json.load(f)
    wl, x, w, sh = _tiny()
    out = orc.layer_unsplit(x, w, sh)["x_out"]
    for (r, c, val) in gold["x_out_samples"]:
        assert out[r, c] == pytest.approx(val, rel=1e-11, abs=1e-12)


def test_error_metric():
    ref = np.array([1.0, -2.0, 0.0, 4.0])
    got = ref + np.array([0.0, 0.02, 0.01, 0.0])
    rms = math.sqrt(21.0 / 4.0)
    assert orc.max_rel_err(got, ref) == pytest.approx(max(0.02 / rms, 0.01 / rms, 0.02 / 2.0 if 2.0 > rms else 0.0))
    assert orc.max_rel_err(ref, ref) == 0.0


def test_bf16_storage_round_trip_is_round_to_nearest_even():
    """The input recipe's bf16 cast: exact halves go to the even neighbour, values survive a round trip."""
    a = np.array([1.0, 1.00390625, 1.01171875, -3.14159, 65504.0, 0.0], dtype=np.float32)
    bits = iso_inputs.f32_to_bf16_bits(a)
    back = iso_inputs.bf16_bits_to_f32(bits)
    # 1 + 2^-8 lies exactly between 1 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies between 1 + 2^-7 (odd) and 1 + 2^-6 (even): goes up
    np.testing.assert_array_equal(back[:3], [1.0, 1.0, 1.015625])
    assert abs(back[3] + 3.14159) <= 2.0 ** -7 and back[4] == 65536.0 and back[5] == 0.0
    np.testing.assert_array_equal(iso_inputs.f32_to_bf16_bits(back), bits)


# ------------------------------------------------------------------ int8 payload (Section 3.2)

def test_quantize_rows_hand_values_and_properties():
    p = np.array([[127.0, -63.5, 0.4, 0.5, 1.5, 2.5, -2.5, 0.0],     # scale 1: ties go to the even code
                  [0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0, 0.0],          # zero row: scale 1, codes 0
                  [-2.54, 1.27, 0.01, 0.0, 0.0, 0.0, 0.0, 0.0]])     # scale 0.02
    codes, scale = orc.quantize_rows(p)
    np.testing.assert_array_equal(codes[0], [127, -64, 0, 0, 2, 2, -2, 0])
    np.testing.assert_array_equal(codes[1], 0)
    assert scale[0] == 1.0 and scale[1] == 1.0 and scale[2] == pytest.approx(0.02, rel=1e-15)
    np.testing.assert_array_equal(codes[2][:3], [-127, 64, 0])        # 63.5 -> 64 (even), 0.5 -> 0 (even)
    x = RNG.standard_normal((9, 64)) * np.logspace(-3, 3, 9)[:, None]
    dq = orc.quant_dequant_rows(x)
    amax = np.abs(x).max(axis=1, keepdims=True)
    assert np.all(np.abs(dq - x) <= amax / 127.0 / 2 * (1 + 1e-12))   # at most half a step
    np.testing.assert_allclose(orc.quant_dequant_rows(dq), dq, rtol=1e-12, atol=0)   # idempotent
    np.testing.assert_array_equal(orc.quantize_rows(-x)[0], -orc.quantize_rows(x)[0])  # symmetric
    # the row maximum is always hit exactly (code +-127)
    assert np.all(np.abs(orc.quantize_rows(x)[0]).max(axis=1) == 127)


def test_fp8_e4m3_format_and_rounding():
    """The 8-bit float of the FP8 projections, against the format's published definition (OCP FP8 E4M3: bias 7,
    three mantissa bits, subnormals, no infinity, S.1111.111 = NaN, largest finite 448) and round-to-nearest-even."""
    v = orc.fp8_e4m3_decode(np.arange(256))
    assert v[0x00] == 0.0 and v[0x38] == 1.0 and v[0x3C] == 1.5 and v[0x40] == 2.0 and v[0xB8] == -1.0
    assert v[0x01] == 2.0 ** -9 and v[0x07] == 7 * 2.0 ** -9 and v[0x08] == 2.0 ** -6       # subnormals, first normal
    assert v[0x7E] == 448.0 and np.isnan(v[0x7F]) and np.isnan(v[0xFF]) and np.nanmax(np.abs(v)) == 448.0
    pos = v[:0x7F]
    assert np.all(np.diff(pos) > 0)                                   # codes are ordered like their values
    fin = v[~np.isnan(v)]
    np.testing.assert_array_equal(orc.fp8_e4m3_round(fin), fin)       # representable values are fixed points
    # halfway cases go to the even mantissa; everything else to the nearer neighbour
    np.testing.assert_array_equal(orc.fp8_e4m3_round([1.0625, 1.1875, 17.0, 19.0, 21.0, 2.0 ** -10, 3 * 2.0 ** -10]),
                                  [1.0, 1.25, 16.0, 20.0, 20.0, 0.0, 2.0 ** -8])
    np.testing.assert_array_equal(orc.fp8_e4m3_round([1.06, 1.07, -0.3, 100.0, 447.0, 500.0, -1e9]),
                                  [1.0, 1.125, -0.3125, 96.0, 448.0, 448.0, -448.0])
    # brute force: the result is the nearest representable value for a dense sweep
    xs = np.concatenate([np.linspace(-460, 460, 20011), np.linspace(-0.05, 0.05, 5003)])
    near = fin[np.argmin(np.abs(xs[:, None] - fin[None, :]), axis=1)]
    got = orc.fp8_e4m3_round(xs)
    ties = np.isclose(np.abs(xs - got), np.abs(xs - near), rtol=0, atol=1e-12)
    assert np.all((got == near) | ties)
    assert np.all(np.abs(got - xs) <= np.maximum(np.abs(xs), 2.0 ** -6) * 2.0 ** -4 + 1e-12)   # half an ulp, relative


def test_fp8_row_quantiser_and_projection():
    """Per-row scales: the largest element of a row maps to 448, a zero row keeps scale 1, scaling a row by a power
    of two changes only its scale, and the FP8 projection stays within the format's error of the exact one."""
    gen = np.random.default_rng(11)
    a = gen.standard_normal((5, 256))
    a[3] = 0.0
    q, s = orc.quantize_rows_fp8(a)
    assert s[3] == 1.0 and np.all(q[3] == 0.0)
    for r in (0, 1, 2, 4):
        assert np.max(np.abs(q[r])) == 448.0
        assert abs(s[r] - np.max(np.abs(a[r].astype(np.float32))) / 448.0) <= 1e-9
        assert np.max(np.abs(q[r] * s[r] - a[r])) <= np.max(np.abs(a[r])) * 2.0 ** -4
    q4, s4 = orc.quantize_rows_fp8(a * 4.0)
    np.testing.assert_array_equal(q4, q)
    np.testing.assert_allclose(s4[[0, 1, 2, 4]], 4.0 * s[[0, 1, 2, 4]], rtol=1e-7)
    w = gen.standard_normal((64, 256)) / 16.0
    exact, got = orc.linear(a, w), orc.linear_fp8(a, w)
    # element errors are below 2^-4 relative and independent: the sum over 256 products errs by ~2^-4 * sqrt(2/3) / ...
    assert 1e-3 < orc.max_rel_err(got, exact) < 0.2
    np.testing.assert_array_equal(got[3], 0.0)
    # quantisation is per row on both sides: a subset of rows or channels gives the same numbers
    np.testing.assert_array_equal(orc.linear_fp8(a[1:3], w[10:20]), got[1:3, 10:20])


def test_fp8_layer_stays_split_invariant_and_near_the_exact_layer():
    wl, x, w, sh = _tiny()
    exact = orc.layer_unsplit(x, w, sh)
    ref = orc.layer_unsplit(x, w, sh, fp8=True)
    assert 1e-3 < orc.max_rel_err(ref["x_out"], exact["x_out"]) < 0.25
    for cuts in (50, [16, 40, 100]):
        got = orc.layer_iso(x, w, sh, cuts, fp8=True)
        assert orc.max_rel_err(got["x_out"], ref["x_out"]) < 1e-12
    rows = [0, 7, 64, 127]
    np.testing.assert_allclose(orc.layer_rows(x, w, sh, rows, fp8=True)["x_out"], ref["x_out"][rows], rtol=0, atol=1e-12)


def test_quantised_layer_stays_split_invariant_and_close_to_the_exact_layer():
    wl, x, w, sh = _tiny()
    exact = orc.layer_unsplit(x, w, sh)["x_out"]
    q = orc.layer_unsplit(x, w, sh, quant=True)["x_out"]
    for s in (1, 37, 64, 127):
        assert orc.max_rel_err(orc.layer_iso(x, w, sh, s, quant=True)["x_out"], q) < 1e-12
    # restricted to some rows the matrix products sum in another order; a partial that sits within 1e-16 of a
    # rounding boundary may then take the neighbouring code: all but a handful of elements agree exactly, and
    # those differ by less than one quantisation step
    r = orc.layer_rows(x, w, sh, [0, 5, 127], quant=True)["x_out"]
    diff = np.abs(r - q[[0, 5, 127]])
    assert np.mean(diff > 1e-9) < 0.01 and diff.max() < np.abs(q).max() / 127.0
    err = orc.max_rel_err(q, exact)
    assert 1e-4 < err < 3e-2          # the payload costs something, but only about half a step of 1/127
