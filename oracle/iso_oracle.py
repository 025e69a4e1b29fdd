"""CPU oracle for the ISO layer-shard prefill.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64 everywhere, no blocking, no fusion.  It shares no code with
the HIP path and must never be imported by the product package: only tests, the
smoke check and the benchmark's cpu_baseline leg may call it.

What is computed (paper, Section 2.2 "gemm overlap": a transformer block is an
attention part -- QKV matrices, attention, o_proj -- and an MLP part -- up/gate
matrices, activation, down matrix -- each ending in a collective; Section 2.1,
tensor parallelism: one device holds a slice of the heads and of the MLP
columns; Section 3.1: the prompt is cut into two chunks along the sequence, each
chunk attends to the KV cache written by the earlier chunk plus itself, and the
result carries no error relative to the unsplit prefill).

The paper does not spell out the block's arithmetic; this build fixes it as the
LLaMA-style pre-norm block: RMSNorm, rotary embedding on rotate-half pairs with
absolute positions, causal softmax attention scaled by 1/sqrt(d) with grouped
query heads, SwiGLU MLP, residual adds.  The tensor-parallel sum over devices is
taken over a world of one device (identity), so the shard's partial output is
what is added to the residual stream.

Pins (tests/test_oracle_pins.py): brute-force masked softmax on tiny inputs,
closed forms for RoPE / SiLU / RMSNorm, a hand-computed two-token layer,
degenerate attention cases, causality, and the split invariance of Section 3.1
for every split point.  The paper prints no worked numerical example, so parity
with the authors' own implementation is unpinned (the result is fixed by the
mathematics above, not by their code).
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Optional, Sequence

import numpy as np


@dataclasses.dataclass(frozen=True)
class LayerShape:
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    rms_eps: float = 1e-6
    rope_base: float = 10000.0


def _f64(a) -> np.ndarray:
    return np.asarray(a, dtype=np.float64)


# ----------------------------------------------------------------------------- steps

def rmsnorm(x, g, eps: float) -> np.ndarray:
    """y[t,:] = x[t,:] / sqrt(mean_h x[t,h]^2 + eps) * g   (norm of the pre-norm block)."""
    x = _f64(x)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * _f64(g)


def linear(a, w) -> np.ndarray:
    """c[t,n] = sum_k a[t,k] w[n,k]   (Section 2.2: QKV, o_proj, up/gate, down matrices)."""
    return _f64(a) @ _f64(w).T


def rope(a, positions, base: float) -> np.ndarray:
    """Rotary embedding on rotate-half pairs (i, i+d/2) at absolute positions.

    a: [t, heads, d]; positions: [t] absolute token indices (a chunk that starts at
    token s uses s, s+1, ... -- Section 3.1 keeps chunk 1 at its place in the prompt).
    theta_i = base^(-2i/d);  out_i = a_i cos(p theta_i) - a_{i+d/2} sin(p theta_i),
    out_{i+d/2} = a_{i+d/2} cos(p theta_i) + a_i sin(p theta_i).
    """
    a = _f64(a)
    d = a.shape[-1]
    half = d // 2
    inv_freq = base ** (-2.0 * np.arange(half, dtype=np.float64) / d)
    ang = _f64(positions)[:, None] * inv_freq[None, :]           # [t, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = a[..., :half], a[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def attention_full(q, k, v) -> np.ndarray:
    """Unsplit causal attention by its definition: whole [T,T] score matrix per head.

    q: [T, nq, d], k, v: [T, nkv, d].  Query head h reads kv head h // (nq // nkv).
    out[t, h, :] = sum_{j<=t} softmax_j(q[t,h].k[j,g] / sqrt(d)) v[j, g, :].
    """
    q, k, v = _f64(q), _f64(k), _f64(v)
    T, nq, d = q.shape
    group = nq // k.shape[1]
    out = np.empty_like(q)
    visible = np.tril(np.ones((T, T), dtype=bool))
    for h in range(nq):
        g = h // group
        s = (q[:, h, :] @ k[:, g, :].T) / math.sqrt(d)
        s = np.where(visible, s, -np.inf)
        s = s - s.max(axis=1, keepdims=True)
        w = np.exp(s)
        w = w / w.sum(axis=1, keepdims=True)
        out[:, h, :] = w @ v[:, g, :]
    return out


def attention_chunk(q, k_cache, v_cache, q_offset: int, kv_len: int) -> np.ndarray:
    """Attention of one chunk over a KV cache (Section 3.1; chunked prefill, Section 2.1).

    q: [Tc, nq, d] are the queries of tokens q_offset .. q_offset+Tc-1.
    k_cache, v_cache: [>=kv_len, nkv, d].  Key j is visible to local row i iff
    j <= q_offset + i and j < kv_len.  Written row by row, one query at a time.
    """
    q, k_cache, v_cache = _f64(q), _f64(k_cache), _f64(v_cache)
    Tc, nq, d = q.shape
    group = nq // k_cache.shape[1]
    out = np.zeros_like(q)
    for i in range(Tc):
        n_vis = min(q_offset + i + 1, kv_len)
        for h in range(nq):
            g = h // group
            scores = k_cache[:n_vis, g, :] @ q[i, h, :] / math.sqrt(d)
            w = np.exp(scores - scores.max())
            out[i, h, :] = (w / w.sum()) @ v_cache[:n_vis, g, :]
    return out


def silu(z) -> np.ndarray:
    z = _f64(z)
    return z / (1.0 + np.exp(-z))


def swiglu(gate_up) -> np.ndarray:
    """a = silu(gate) * up with gate = first half, up = second half of the last axis
    (Section 2.2: the activation between the up/gate and down matrices)."""
    gu = _f64(gate_up)
    f = gu.shape[-1] // 2
    return silu(gu[..., :f]) * gu[..., f:]


def quantize_rows(p):
    """Int8 payload of a communication point (Section 3.2, "communication dominates": the data sent is
    quantised to int8).  The paper does not give the quantiser; this build fixes it as symmetric per token
    row: scale = max|p| / 127 (1 for an all-zero row), code = p / scale rounded to nearest, ties to even,
    clipped to [-127, 127].  Returns (codes int8 [T,H], scales float64 [T])."""
    p = _f64(p)
    amax = np.max(np.abs(p), axis=-1)
    scale = np.where(amax > 0, amax / 127.0, 1.0)
    codes = np.clip(np.rint(p / scale[..., None]), -127, 127).astype(np.int8)
    return codes, scale


def quant_dequant_rows(p):
    """What a receiver of the int8 payload adds to its residual stream: code * scale."""
    codes, scale = quantize_rows(p)
    return codes.astype(np.float64) * scale[..., None]


def _comm(p, quant: bool):
    """All-reduce over a world of one rank: the identity, optionally through the int8 payload."""
    return quant_dequant_rows(p) if quant else p


# ----------------------------------------------------------------------------- fp8 projections

FP8_MAX = 448.0          # largest finite value of the 8-bit format below


def fp8_e4m3_decode(code) -> np.ndarray:
    """Value of an OCP FP8 E4M3 byte: 1 sign, 4 exponent (bias 7), 3 mantissa bits; exponent 0 is
    subnormal (m/8 * 2^-6); S.1111.111 is NaN, there is no infinity, the largest finite value is 448."""
    code = np.asarray(code, dtype=np.int64)
    sign = np.where(code & 0x80, -1.0, 1.0)
    e = (code >> 3) & 0xF
    m = (code & 7).astype(np.float64)
    val = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7.0))
    val = np.where((e == 15) & ((code & 7) == 7), np.nan, val)
    return sign * val


def fp8_e4m3_round(x) -> np.ndarray:
    """x rounded to the nearest FP8 E4M3 value, ties to the even mantissa, magnitudes above 448 clipped to
    448.  Returned as float64 values (not codes)."""
    x = _f64(x)
    a = np.minimum(np.abs(x), FP8_MAX)
    with np.errstate(divide="ignore"):
        e = np.floor(np.log2(np.where(a > 0, a, 1.0)))
    e = np.clip(e, -6.0, 8.0)                 # below 2^-6 the spacing stays that of the subnormals
    quantum = 2.0 ** (e - 3.0)
    return np.sign(x) * np.minimum(np.rint(a / quantum) * quantum, FP8_MAX)


def quantize_rows_fp8(a):
    """Per-row FP8 quantisation of a projection operand (Section 4.1: the paper runs its matrix products in
    8 bits; this build uses the 8-bit float the target's matrix cores take, with one scale per row).
    In float32, as the device does it: amax = max|row|, inv = 448 / amax, value = fp8(a * inv),
    scale = amax / 448 (inv = scale = 1 for an all-zero row).  Returns (fp8 values as float64 [T,K],
    scales float64 [T]); the represented row is value * scale."""
    a32 = np.asarray(a, dtype=np.float64).astype(np.float32)
    amax = np.max(np.abs(a32), axis=-1)
    nz = amax > 0
    inv = np.where(nz, np.float32(FP8_MAX) / np.where(nz, amax, np.float32(1)), np.float32(1)).astype(np.float32)
    scale = np.where(nz, amax / np.float32(FP8_MAX), np.float32(1)).astype(np.float32)
    scaled = (a32 * inv[..., None]).astype(np.float32)
    return fp8_e4m3_round(scaled), scale.astype(np.float64)


def linear_fp8(a, w) -> np.ndarray:
    """a w^T with both operands quantised per row to FP8 (rows of w = output channels); exact product of
    the quantised values, then the two row scales."""
    aq, sa = quantize_rows_fp8(a)
    wq, sw = quantize_rows_fp8(w)
    return (aq @ wq.T) * sa[:, None] * sw[None, :]


# ----------------------------------------------------------------------------- layer

def _split_qkv(qkv: np.ndarray, sh: LayerShape):
    t = qkv.shape[0]
    nq, nkv, d = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    q = qkv[:, : nq * d].reshape(t, nq, d)
    k = qkv[:, nq * d: (nq + nkv) * d].reshape(t, nkv, d)
    v = qkv[:, (nq + nkv) * d:].reshape(t, nkv, d)
    return q, k, v


def _lin(a, w, fp8: bool) -> np.ndarray:
    """A projection of the layer: exact, or with both operands quantised per row to FP8 (Section 4.1)."""
    return linear_fp8(a, w) if fp8 else linear(a, w)


def mlp_partial(x1: np.ndarray, w: Dict[str, np.ndarray], sh: LayerShape, fp8: bool = False) -> np.ndarray:
    """Row-parallel partial of the MLP block: down(swiglu(gate_up(rmsnorm(x1))))."""
    y2 = rmsnorm(x1, w["g_mlp"], sh.rms_eps)
    a = swiglu(_lin(y2, w["w_gate_up"], fp8))
    return _lin(a, w["w_down"], fp8)


def _mlp_block(x1: np.ndarray, w: Dict[str, np.ndarray], sh: LayerShape, quant: bool = False,
               fp8: bool = False) -> np.ndarray:
    pm = mlp_partial(x1, w, sh, fp8)     # all-reduce over one device = identity
    return x1 + _comm(pm, quant)


def layer_unsplit(x, w: Dict[str, np.ndarray], sh: LayerShape, quant: bool = False,
                  fp8: bool = False) -> Dict[str, np.ndarray]:
    """One decoder-layer shard over the whole prompt (the pipeline ISO is compared with).
    quant=True sends both partials through the int8 payload of Section 3.2 (per-row quantisation acts on
    each token separately, so it commutes with the chunking).  fp8=True runs the four projections on
    operands quantised per row to FP8 (also per token, so it commutes with the chunking too)."""
    x = _f64(x)
    T = x.shape[0]
    pos = np.arange(T)
    y = rmsnorm(x, w["g_attn"], sh.rms_eps)
    q, k, v = _split_qkv(_lin(y, w["w_qkv"], fp8), sh)
    q = rope(q, pos, sh.rope_base)
    k = rope(k, pos, sh.rope_base)
    o = attention_full(q, k, v).reshape(T, sh.n_q_heads * sh.head_dim)
    pa = _lin(o, w["w_o"], fp8)          # row-parallel partial
    x1 = x + _comm(pa, quant)
    return {"x_out": _mlp_block(x1, w, sh, quant, fp8), "k_cache": k, "v_cache": v, "x1": x1, "attn": o, "pa": pa}


def layer_iso(x, w: Dict[str, np.ndarray], sh: LayerShape, split, quant: bool = False,
              fp8: bool = False) -> Dict[str, np.ndarray]:
    """The same layer as consecutive chunks (Section 3.1: two chunks; Section 6: finer cuts).

    `split` is one cut point or an ascending list of cut points strictly inside the prompt.  Chunk c
    writes its K/V rows into the cache and attends to the cache up to its own last row; everything
    else is per token.
    """
    x = _f64(x)
    T = x.shape[0]
    cuts = [int(split)] if np.isscalar(split) else [int(c) for c in split]
    edges = [0] + cuts + [T]
    if any(b <= a for a, b in zip(edges[:-1], edges[1:])):
        raise ValueError("cut points must be ascending and lie strictly inside the prompt")
    k_cache = np.zeros((T, sh.n_kv_heads, sh.head_dim))
    v_cache = np.zeros((T, sh.n_kv_heads, sh.head_dim))
    x_out = np.empty_like(x)
    x1_all = np.empty_like(x)
    for lo, hi in zip(edges[:-1], edges[1:]):
        xc = x[lo:hi]
        pos = np.arange(lo, hi)
        y = rmsnorm(xc, w["g_attn"], sh.rms_eps)
        q, k, v = _split_qkv(_lin(y, w["w_qkv"], fp8), sh)
        q = rope(q, pos, sh.rope_base)
        k_cache[lo:hi] = rope(k, pos, sh.rope_base)
        v_cache[lo:hi] = v
        o = attention_chunk(q, k_cache, v_cache, q_offset=lo, kv_len=hi)
        pa = _lin(o.reshape(hi - lo, -1), w["w_o"], fp8)
        x1 = xc + _comm(pa, quant)
        x1_all[lo:hi] = x1
        x_out[lo:hi] = _mlp_block(x1, w, sh, quant, fp8)
    return {"x_out": x_out, "k_cache": k_cache, "v_cache": v_cache, "x1": x1_all}


def token_cost(sh: LayerShape, T: int, attn_flop_cost: float) -> np.ndarray:
    """Cost of each prompt position in projection-flop units (Section 6: the later half of the
    sequence is dearer because its attention reads more keys).

    Position i pays the projections (the same for every token) plus attention over i + 1 keys, two
    products of 2 * d flops per query head and key, weighted by how much dearer an attention flop is
    than a projection flop.
    """
    nq, nkv, d, H, F = sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.hidden, sh.ffn
    proj = 2.0 * H * (nq + 2 * nkv) * d + 2.0 * H * nq * d + 6.0 * H * F
    keys = np.arange(1, T + 1, dtype=np.float64)
    return proj + attn_flop_cost * 4.0 * nq * d * keys


def balanced_cuts(sh: LayerShape, T: int, n_chunks: int, attn_flop_cost: float) -> np.ndarray:
    """Real-valued cut positions t_j (j = 1 .. n_chunks-1) at which the cumulative cost of the prompt,
    taken as a continuous function of the position, reaches j / n_chunks of its total: chunks of
    equal cost instead of equal length (Section 6)."""
    c = np.concatenate([[0.0], np.cumsum(token_cost(sh, T, attn_flop_cost))])
    targets = c[-1] * np.arange(1, n_chunks) / n_chunks
    return np.interp(targets, c, np.arange(T + 1, dtype=np.float64))


def layer_rows(x, w: Dict[str, np.ndarray], sh: LayerShape, rows: Sequence[int], quant: bool = False,
               fp8: bool = False) -> Dict[str, np.ndarray]:
    """Exact output rows `rows` of the layer, without computing the others.

    Output row p depends on x[p] and on the K/V rows 0..p only, so K/V are computed
    for every token and the rest (q, attention, o_proj, MLP) for the listed rows.
    This is the definition restricted to some rows, not an approximation.
    """
    x = _f64(x)
    T = x.shape[0]
    nq, nkv, d = sh.n_q_heads, sh.n_kv_heads, sh.head_dim
    rows = np.asarray(list(rows), dtype=np.int64)
    y = rmsnorm(x, w["g_attn"], sh.rms_eps)
    w_qkv = _f64(w["w_qkv"])
    kv = _lin(y, w_qkv[nq * d:], fp8)
    k = rope(kv[:, : nkv * d].reshape(T, nkv, d), np.arange(T), sh.rope_base)
    v = kv[:, nkv * d:].reshape(T, nkv, d)
    q = rope(_lin(y[rows], w_qkv[: nq * d], fp8).reshape(len(rows), nq, d), rows, sh.rope_base)
    o = np.empty((len(rows), nq, d))
    for r, p in enumerate(rows):
        o[r] = attention_chunk(q[r:r + 1], k, v, q_offset=int(p), kv_len=int(p) + 1)[0]
    pa = _lin(o.reshape(len(rows), nq * d), w["w_o"], fp8)
    x1 = x[rows] + _comm(pa, quant)
    return {"x_out": _mlp_block(x1, w, sh, quant, fp8), "k_cache": k, "v_cache": v, "x1": x1, "rows": rows, "pa": pa}


# ----------------------------------------------------------------------------- metric

def max_rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)): element-wise relative error with the
    denominator floored at the tensor's RMS so that near-zero references do not dominate."""
    got, ref = _f64(got), _f64(ref)
    rms = math.sqrt(float(np.mean(ref * ref))) if ref.size else 0.0
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den)) if ref.size else 0.0
