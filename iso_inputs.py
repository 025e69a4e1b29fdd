"""Seeded synthetic inputs for the ISO layer-shard prefill.

This module only draws random tensors and names workload shapes.  It holds none
of the method's arithmetic and is the only code shared by the CPU oracle's
callers and the HIP path's callers: both receive exactly the same tensors.

Workloads follow the model classes the paper evaluates (Section 4.1: dense ~30B
MHA and ~70B GQA models, batch size 1, prompts of 1k-128k tokens) cut into one
tensor-parallel shard (Section 2.1, tensor parallelism): the shard keeps
`n_q_heads`/`n_kv_heads` local heads and `ffn` local MLP columns, and the full
hidden width.  The paper's weights and prompts are proprietary, so values are
synthetic: hidden states N(0,1), matrices N(0, 1/fan_in) with fan_in the
contraction length as stored in the shard, RMSNorm gains 1 + 0.1*N(0,1).
"""
from __future__ import annotations

import dataclasses
from typing import Dict

import numpy as np


# ---- bf16 storage format: the upper 16 bits of an IEEE float32, rounded to nearest even ------------
# (format conversion for input preparation; arrays of bf16 values are held as uint16 bit patterns)

def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """fp32 draw -> storage array of the workload dtype ("f32": float32, "bf16": uint16 bit patterns)."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    return f32_to_bf16_bits(a)


def to_f64(a: np.ndarray, dtype: str) -> np.ndarray:
    """Exact float64 values of a storage array (what both the oracle and the GPU see)."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    return bf16_bits_to_f32(a).astype(np.float64)


def np_storage_dtype(dtype: str):
    return np.float32 if dtype == "f32" else np.uint16


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    seq: int
    split: int
    dtype: str          # "f32" or "bf16"
    n_layers: int = 1
    rms_eps: float = 1e-6
    rope_base: float = 10000.0

    @property
    def n_qkv(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def gemm_flops(self, tokens: int | None = None) -> float:
        """2*M*N*K over the four projections of one layer."""
        t = self.seq if tokens is None else tokens
        h, d, f = self.hidden, self.head_dim, self.ffn
        per_tok = 2 * h * self.n_qkv + 2 * self.n_q_heads * d * h + 4 * h * f + 2 * f * h
        return float(per_tok) * t

    def attn_flops(self, q_offset: int = 0, tc: int | None = None) -> float:
        """4*d*nq per visible (query, key) pair of a causal chunk."""
        tc = self.seq if tc is None else tc
        pairs = tc * q_offset + tc * (tc + 1) // 2
        return 4.0 * self.head_dim * self.n_q_heads * pairs

    def layer_flops(self) -> float:
        return self.gemm_flops() + self.attn_flops()


def split_point(seq: int, frac: float) -> int:
    """Split used for a fractional split request: nearest multiple of 32."""
    return int(round(frac * seq / 32.0)) * 32


WORKLOADS: Dict[str, Workload] = {
    w.name: w
    for w in [
        # small case the oracle finishes in well under a second
        Workload("tiny_f32", 256, 4, 4, 64, 688, 128, 64, "f32"),
        # ~30B MHA model, one TP=4 shard, 2k prompt
        Workload("30b_tp4_2k", 6656, 13, 13, 128, 4480, 2048, 1024, "bf16"),
        # ~70B GQA model, one TP=8 shard, 4k prompt
        Workload("70b_tp8_4k", 8192, 8, 1, 128, 3584, 4096, 2048, "bf16"),
        # ~70B GQA model, one TP=4 shard, 8k prompt (split swept in tests/bench)
        Workload("70b_tp4_8k", 8192, 16, 2, 128, 7168, 8192, 4096, "bf16"),
        # ~70B GQA model, one TP=8 shard, full 80-layer stack, 16k prompt
        Workload("70b_tp8_16k_stack", 8192, 8, 1, 128, 3584, 16384, 8192, "bf16", n_layers=80),
        # the long prompts of the paper's Table 1 at the same shard: attention grows from a quarter to most of the
        # flops; the cut leaves the first chunk the longer one (Section 6)
        Workload("70b_tp8_32k", 8192, 8, 1, 128, 3584, 32768, 18432, "bf16"),
        Workload("70b_tp8_64k", 8192, 8, 1, 128, 3584, 65536, 37888, "bf16"),
        Workload("70b_tp8_128k", 8192, 8, 1, 128, 3584, 131072, 77824, "bf16"),
    ]
}


def _randn(gen: np.random.Generator, *shape: int) -> np.ndarray:
    return gen.standard_normal(shape, dtype=np.float32)


def make_layer(hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int, ffn: int,
               seed: int, dtype: str) -> Dict[str, np.ndarray]:
    """Random weights of one layer shard, as storage arrays of `dtype` ("f32" or "bf16").

    Draw order: w_qkv, w_o, w_gate_up, w_down, g_attn, g_mlp (fp32 draws from numpy's PCG64 seeded with
    `seed`, then a round-to-nearest-even cast for bf16).
    """
    gen = np.random.default_rng(seed)
    n_qkv = (n_q_heads + 2 * n_kv_heads) * head_dim
    nqd = n_q_heads * head_dim
    w = {
        "w_qkv": _randn(gen, n_qkv, hidden) * np.float32(hidden ** -0.5),
        "w_o": _randn(gen, hidden, nqd) * np.float32(nqd ** -0.5),
        "w_gate_up": _randn(gen, 2 * ffn, hidden) * np.float32(hidden ** -0.5),
        "w_down": _randn(gen, hidden, ffn) * np.float32(ffn ** -0.5),
        "g_attn": np.float32(1.0) + np.float32(0.1) * _randn(gen, hidden),
        "g_mlp": np.float32(1.0) + np.float32(0.1) * _randn(gen, hidden),
    }
    return {k: store(v, dtype) for k, v in w.items()}


def make_hidden(seq: int, hidden: int, seed: int, dtype: str) -> np.ndarray:
    """Input hidden states x[seq, hidden] ~ N(0,1)."""
    gen = np.random.default_rng(seed + 7919)
    return store(_randn(gen, seq, hidden), dtype)


def make_workload_inputs(w: Workload, seed: int = 0, layer: int = 0):
    """(x, weights) for one layer of a named workload; layer l uses seed 1000*seed + l."""
    weights = make_layer(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, 1000 * seed + layer, w.dtype)
    x = make_hidden(w.seq, w.hidden, seed, w.dtype)
    return x, weights


def make_workload_inputs_layer(w: Workload, seed: int = 0, layer: int = 0) -> Dict[str, np.ndarray]:
    """The weights of layer `layer` of a named workload alone (same draws as make_workload_inputs)."""
    return make_layer(w.hidden, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ffn, 1000 * seed + layer, w.dtype)


def make_qkv_cache(tc: int, kv_len: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                   seed: int, dtype: str):
    """Random q[tc, nq, d], k[kv_len, nkv, d], v[kv_len, nkv, d] for attention-only tests."""
    gen = np.random.default_rng(seed)
    q = store(_randn(gen, tc, n_q_heads, head_dim), dtype)
    k = store(_randn(gen, kv_len, n_kv_heads, head_dim), dtype)
    v = store(_randn(gen, kv_len, n_kv_heads, head_dim), dtype)
    return q, k, v


def randn(shape, seed: int, dtype: str, scale: float = 1.0) -> np.ndarray:
    """A seeded N(0, scale^2) storage array for single-step tests."""
    gen = np.random.default_rng(seed)
    return store(_randn(gen, *shape) * np.float32(scale), dtype)


def sample_rows(seq: int, split: int, n: int, seed: int = 0):
    """Row set for sampled parity at full sizes: chunk edges plus uniform draws, half per chunk."""
    fixed = {0, 1, seq - 1}
    if 0 < split < seq:
        fixed |= {split - 1, split, min(split + 1, seq - 1)}
    gen = np.random.default_rng(seed + 104729)
    rows = set(r for r in fixed if 0 <= r < seq)
    s = split if 0 < split < seq else seq // 2
    while len(rows) < min(n, seq):
        lo, hi = (0, s) if len(rows) % 2 == 0 else (s, seq)
        if hi <= lo:
            lo, hi = 0, seq
        rows.add(int(gen.integers(lo, hi)))
    return sorted(rows)
