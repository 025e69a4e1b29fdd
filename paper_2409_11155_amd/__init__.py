"""Python binding of libiso: argument marshalling only.

Every step of the ISO layer-shard prefill runs inside the HIP kernels of libiso.so; this module turns
numpy arrays, device buffers and streams into the plain pointers and sizes of the C ABI (include/iso.h)
and turns error codes into exceptions.  There is no fallback: if the library cannot be loaded, every
call raises.

Device buffers and streams come from the library itself (DeviceArray, Stream), so a process needs no
other GPU framework.  Objects from other frameworks still work where a pointer is expected: anything with
a `data_ptr()` method is taken as a device buffer and anything with a `cuda_stream` attribute as a stream.
Import this package before any other library that bundles its own HIP runtime: the first HIP runtime
loaded into the process is the one libiso binds to.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Dict, Optional, Sequence

import numpy as np

from . import build as _build

ISO_OK = 0
ISO_ERR_NULL, ISO_ERR_SHAPE, ISO_ERR_DTYPE, ISO_ERR_SPLIT, ISO_ERR_WORKSPACE, ISO_ERR_HIP = -1, -2, -3, -4, -5, -6
ISO_F32, ISO_BF16 = 0, 1
ISO_COMM_NONE, ISO_COMM_D2H, ISO_COMM_D2H_INT8 = 0, 1, 2
ISO_SCHED_OVERLAP, ISO_SCHED_SERIAL, ISO_SCHED_STREAM_PER_CHUNK = 0, 1, 2
ISO_MAX_CHUNKS = 8
ISO_FLAG_SIMPLE_GEMM, ISO_FLAG_SIMPLE_ATTN, ISO_FLAG_GEMM_STAGED, ISO_FLAG_NO_FUSE, ISO_FLAG_ATTN_STAGED = 1, 2, 4, 8, 16
ISO_FLAG_NO_STREAMK = 32
ISO_FLAG_FP8_GEMM = 64

EXPORTS = [
    "iso_validate_cfg", "iso_plan_chunks", "iso_plan_split", "iso_plan_chunk_count", "iso_stack_prefill_chunks", "iso_create", "iso_destroy", "iso_sync", "iso_last_error",
    "iso_layer_prefill", "iso_stack_prefill", "iso_attn_chunk", "iso_gemm_rowpar", "iso_rmsnorm",
    "iso_residual_rmsnorm", "iso_rope_kv_write", "iso_swiglu", "iso_set_flags", "iso_host_sink",
    "iso_timing_enable", "iso_timing_read",
    "iso_device_count", "iso_device_sync", "iso_dev_alloc", "iso_dev_free", "iso_dev_fill", "iso_host_alloc",
    "iso_host_free", "iso_copy_h2d", "iso_copy_d2h", "iso_copy_d2h_async", "iso_set_gemm_segments", "iso_quantize_rows_fp8", "iso_rmsnorm_fp8", "iso_gemm_fp8", "iso_gemm_launch_plan", "iso_copy_d2d", "iso_stream_create", "iso_stream_destroy",
    "iso_gemm_rowpar_static", "iso_streamk_status_word",
]
KERNEL_KINDS = ["gemm_qkv", "gemm_o", "gemm_gate_up", "gemm_down", "attn", "rmsnorm", "resid_norm", "residual",
                "rope_kv", "swiglu", "comm", "quant"]
DTYPE_BYTES = {"f32": 4, "bf16": 2, "u8": 1}
_NP_STORAGE = {"f32": np.float32, "bf16": np.uint16, "u8": np.uint8}


class IsoCfg(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int), ("n_q_heads", ctypes.c_int), ("n_kv_heads", ctypes.c_int),
                ("head_dim", ctypes.c_int), ("ffn", ctypes.c_int), ("rms_eps", ctypes.c_float),
                ("rope_base", ctypes.c_float), ("dtype", ctypes.c_int), ("max_seq", ctypes.c_int)]


class IsoWeights(ctypes.Structure):
    _fields_ = [("w_qkv", ctypes.c_void_p), ("w_o", ctypes.c_void_p), ("w_gate_up", ctypes.c_void_p),
                ("w_down", ctypes.c_void_p), ("g_attn", ctypes.c_void_p), ("g_mlp", ctypes.c_void_p),
                ("w_qkv_f8", ctypes.c_void_p), ("w_o_f8", ctypes.c_void_p), ("w_gate_up_f8", ctypes.c_void_p),
                ("w_down_f8", ctypes.c_void_p), ("s_qkv", ctypes.c_void_p), ("s_o", ctypes.c_void_p),
                ("s_gate_up", ctypes.c_void_p), ("s_down", ctypes.c_void_p)]


class IsoPlan(ctypes.Structure):
    _fields_ = [("n_chunks", ctypes.c_int), ("q_offset", ctypes.c_int * 2), ("n_tokens", ctypes.c_int * 2),
                ("kv_len", ctypes.c_int * 2), ("comm_bytes", ctypes.c_size_t * 2),
                ("workspace_bytes", ctypes.c_size_t)]


class IsoError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libiso error {code}: {msg}")
        self.code = code


_lib: Optional[ctypes.CDLL] = None


def lib_path() -> str:
    return _build.LIB_PATH


def load() -> ctypes.CDLL:
    """Loads libiso.so (building it once if no built library is present)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build(verbose=False)
    lib = ctypes.CDLL(_build.LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    pvp = ctypes.POINTER(vp)
    lib.iso_last_error.restype = ctypes.c_char_p
    lib.iso_last_error.argtypes = []
    lib.iso_validate_cfg.argtypes = [ctypes.POINTER(IsoCfg)]
    lib.iso_plan_chunks.argtypes = [ctypes.POINTER(IsoCfg), ci, ci, ctypes.POINTER(IsoPlan)]
    lib.iso_plan_chunk_count.argtypes = [ctypes.POINTER(IsoCfg), ci, ctypes.POINTER(ci)]
    lib.iso_plan_split.argtypes = [ctypes.POINTER(IsoCfg), ci, ci, ctypes.c_double, ctypes.POINTER(ci)]
    lib.iso_create.argtypes = [pvp, ctypes.POINTER(IsoCfg), vp, vp]
    lib.iso_destroy.argtypes = [vp]
    lib.iso_sync.argtypes = [vp]
    lib.iso_set_flags.argtypes = [vp, ci]
    lib.iso_host_sink.argtypes = [vp]
    lib.iso_host_sink.restype = vp
    lib.iso_layer_prefill.argtypes = [vp, ctypes.POINTER(IsoWeights), vp, vp, vp, ci, ci, ci, ci]
    lib.iso_stack_prefill.argtypes = [vp, ctypes.POINTER(IsoWeights), ci, vp, vp, vp, ci, ci, ci, ci]
    lib.iso_stack_prefill_chunks.argtypes = [vp, ctypes.POINTER(IsoWeights), ci, vp, vp, vp, ci, ctypes.POINTER(ci), ci,
                                             ci, ci]
    lib.iso_attn_chunk.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, vp]
    lib.iso_gemm_rowpar.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp, vp]
    lib.iso_gemm_rowpar_static.argtypes = [vp, vp, vp, vp, ci, ci, ci, vp]
    lib.iso_streamk_status_word.argtypes = [vp]
    lib.iso_streamk_status_word.restype = ctypes.POINTER(ctypes.c_uint)
    lib.iso_rmsnorm.argtypes = [vp, vp, vp, vp, ci, vp]
    lib.iso_residual_rmsnorm.argtypes = [vp, vp, vp, vp, vp, ci, vp]
    lib.iso_rope_kv_write.argtypes = [vp, vp, vp, vp, ci, ci, vp]
    lib.iso_swiglu.argtypes = [vp, vp, vp, ci, vp]
    lib.iso_timing_enable.argtypes = [vp, ci]
    lib.iso_timing_read.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ci)]
    lib.iso_device_count.argtypes = [ctypes.POINTER(ci)]
    lib.iso_device_sync.argtypes = []
    lib.iso_dev_alloc.argtypes = [pvp, sz]
    lib.iso_dev_free.argtypes = [vp]
    lib.iso_dev_fill.argtypes = [vp, ci, sz]
    lib.iso_host_alloc.argtypes = [pvp, sz]
    lib.iso_host_free.argtypes = [vp]
    lib.iso_copy_h2d.argtypes = [vp, vp, sz]
    lib.iso_copy_d2h.argtypes = [vp, vp, sz]
    lib.iso_copy_d2h_async.argtypes = [vp, vp, sz, vp]
    lib.iso_set_gemm_segments.argtypes = [vp, ci]
    lib.iso_gemm_launch_plan.argtypes = [ci, ci, ci, ci, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ci)]
    lib.iso_quantize_rows_fp8.argtypes = [vp, vp, ci, ci, vp, vp, vp]
    lib.iso_rmsnorm_fp8.argtypes = [vp, vp, vp, vp, vp, vp, ci, vp]
    lib.iso_gemm_fp8.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, vp]
    lib.iso_copy_d2d.argtypes = [vp, vp, sz]
    lib.iso_stream_create.argtypes = [pvp]
    lib.iso_stream_destroy.argtypes = [vp]
    for name in EXPORTS:
        if name not in ("iso_last_error", "iso_host_sink", "iso_streamk_status_word"):
            getattr(lib, name).restype = ci
    _lib = lib
    return lib


def last_error() -> str:
    return load().iso_last_error().decode()


def _check(code: int) -> None:
    if code != ISO_OK:
        raise IsoError(code, last_error())


def device_count() -> int:
    n = ctypes.c_int(0)
    _check(load().iso_device_count(ctypes.byref(n)))
    return n.value


def device_sync() -> None:
    _check(load().iso_device_sync())


def make_cfg(hidden: int, n_q_heads: int, n_kv_heads: int, head_dim: int, ffn: int, dtype, max_seq: int,
             rms_eps: float = 1e-6, rope_base: float = 10000.0) -> IsoCfg:
    if isinstance(dtype, str):
        dtype = {"f32": ISO_F32, "bf16": ISO_BF16}[dtype]
    return IsoCfg(hidden, n_q_heads, n_kv_heads, head_dim, ffn, rms_eps, rope_base, int(dtype), max_seq)


def validate_cfg(cfg: IsoCfg) -> int:
    return load().iso_validate_cfg(ctypes.byref(cfg))


def plan_chunks(cfg: IsoCfg, T: int, split: int) -> IsoPlan:
    plan = IsoPlan()
    _check(load().iso_plan_chunks(ctypes.byref(cfg), T, split, ctypes.byref(plan)))
    return plan


ISO_GEMM_TILE_256, ISO_GEMM_TILE_128, ISO_GEMM_STREAMK, ISO_GEMM_STAGED, ISO_GEMM_SIMPLE = 1, 3, 6, 100, 101


def gemm_launch_plan(M: int, N: int, K: int, num_cu: int = 256):
    """(kind, team, grid) of the bf16 projection kernel chosen for these sizes."""
    kind, team, grid = ctypes.c_int(), ctypes.c_int(), ctypes.c_int()
    _check(load().iso_gemm_launch_plan(M, N, K, num_cu, ctypes.byref(kind), ctypes.byref(team), ctypes.byref(grid)))
    return kind.value, team.value, grid.value


def plan_chunk_count(cfg: IsoCfg, T: int) -> int:
    n = ctypes.c_int()
    _check(load().iso_plan_chunk_count(ctypes.byref(cfg), T, ctypes.byref(n)))
    return n.value


def plan_split(cfg: IsoCfg, T: int, n_chunks: int, attn_flop_cost: float = 0.0) -> List[int]:
    """Cut points for n_chunks chunks of equal estimated cost (attn_flop_cost <= 0: the library's default)."""
    out = (ctypes.c_int * max(1, n_chunks - 1))()
    _check(load().iso_plan_split(ctypes.byref(cfg), T, n_chunks, float(attn_flop_cost), out if n_chunks > 1 else None))
    return [int(out[i]) for i in range(n_chunks - 1)]


# ------------------------------------------------------------------------------ buffers and streams

class DeviceArray:
    """A device allocation with a shape and an element type ("f32" or "bf16").  bf16 values travel to and
    from the host as uint16 bit patterns (numpy has no bf16)."""

    def __init__(self, shape, dtype: str, fill_byte: Optional[int] = None):
        self._lib = load()
        self.shape = tuple(int(s) for s in (shape if isinstance(shape, (tuple, list)) else (shape,)))
        self.dtype = dtype
        self.nbytes = int(np.prod(self.shape, dtype=np.int64)) * DTYPE_BYTES[dtype]
        p = ctypes.c_void_p()
        _check(self._lib.iso_dev_alloc(ctypes.byref(p), self.nbytes))
        self.ptr = p.value
        if fill_byte is not None:
            self.fill(fill_byte)

    @classmethod
    def from_numpy(cls, a: np.ndarray, dtype: str) -> "DeviceArray":
        a = np.ascontiguousarray(a)
        if a.dtype != _NP_STORAGE[dtype]:
            raise TypeError(f"{dtype} arrays are stored as {_NP_STORAGE[dtype].__name__}, got {a.dtype}")
        out = cls(a.shape, dtype)
        out.upload(a)
        return out

    def upload(self, a: np.ndarray) -> None:
        a = np.ascontiguousarray(a)
        if a.nbytes != self.nbytes:
            raise ValueError("size mismatch")
        _check(self._lib.iso_copy_h2d(self.ptr, a.ctypes.data, self.nbytes))

    def numpy(self) -> np.ndarray:
        out = np.empty(self.shape, dtype=_NP_STORAGE[self.dtype])
        _check(self._lib.iso_copy_d2h(out.ctypes.data, self.ptr, self.nbytes))
        return out

    def fill(self, byte_value: int) -> None:
        _check(self._lib.iso_dev_fill(self.ptr, byte_value, self.nbytes))

    def copy_from(self, other: "DeviceArray") -> None:
        if other.nbytes != self.nbytes:
            raise ValueError("size mismatch")
        _check(self._lib.iso_copy_d2d(self.ptr, other.ptr, self.nbytes))

    def clone(self) -> "DeviceArray":
        out = DeviceArray(self.shape, self.dtype)
        out.copy_from(self)
        return out

    def data_ptr(self) -> int:
        return self.ptr

    def free(self) -> None:
        if getattr(self, "ptr", None):
            self._lib.iso_dev_free(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class PinnedArray:
    """Pinned host memory viewed as a numpy array (for the communication stand-in's destination)."""

    def __init__(self, shape, dtype: str):
        self._lib = load()
        self.shape = tuple(shape)
        self.dtype = dtype
        self.nbytes = int(np.prod(self.shape, dtype=np.int64)) * DTYPE_BYTES[dtype]
        p = ctypes.c_void_p()
        _check(self._lib.iso_host_alloc(ctypes.byref(p), self.nbytes))
        self.ptr = p.value
        buf = (ctypes.c_byte * self.nbytes).from_address(self.ptr)
        self.array = np.frombuffer(buf, dtype=_NP_STORAGE[dtype]).reshape(self.shape)

    def free(self) -> None:
        if getattr(self, "ptr", None):
            self.array = None
            self._lib.iso_host_free(self.ptr)
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Stream:
    """A non-blocking HIP stream of default priority."""

    def __init__(self):
        self._lib = load()
        p = ctypes.c_void_p()
        _check(self._lib.iso_stream_create(ctypes.byref(p)))
        self.handle = p.value

    def destroy(self) -> None:
        if getattr(self, "handle", None):
            self._lib.iso_stream_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if hasattr(t, "is_contiguous") and not t.is_contiguous():
        raise ValueError("libiso takes contiguous buffers")
    return t.data_ptr()


def copy_d2h_async(dst: "PinnedArray", src: "DeviceArray", nbytes: int, stream) -> None:
    """Asynchronous device-to-host copy of the first nbytes of src into pinned memory, in `stream`."""
    _check(load().iso_copy_d2h_async(dst.ptr, src.ptr, int(nbytes), _stream_handle(stream)))


def _stream_handle(s) -> Optional[int]:
    if s is None:
        return None
    if isinstance(s, Stream):
        return s.handle
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream or None
    return int(s) or None


def pack_weights(w: Dict[str, object]) -> IsoWeights:
    opt = [_ptr(w[k]) if k in w else None
           for k in ("w_qkv_f8", "w_o_f8", "w_gate_up_f8", "w_down_f8", "s_qkv", "s_o", "s_gate_up", "s_down")]
    return IsoWeights(_ptr(w["w_qkv"]), _ptr(w["w_o"]), _ptr(w["w_gate_up"]), _ptr(w["w_down"]),
                      _ptr(w["g_attn"]), _ptr(w["g_mlp"]), *opt)


def upload_weights(w: Dict[str, np.ndarray], dtype: str) -> Dict[str, DeviceArray]:
    return {k: DeviceArray.from_numpy(v, dtype) for k, v in w.items()}


class Context:
    """Owns an iso_ctx.  `stream0`/`stream1`: Stream objects (created here if omitted)."""

    def __init__(self, cfg: IsoCfg, stream0=None, stream1=None, two_streams: bool = True):
        self._lib = load()
        self.cfg = cfg
        if stream0 is None:
            stream0 = Stream()
        if stream1 is None:
            stream1 = Stream() if two_streams else stream0
        self.stream0, self.stream1 = stream0, stream1   # keep the streams alive
        handle = ctypes.c_void_p()
        _check(self._lib.iso_create(ctypes.byref(handle), ctypes.byref(cfg), _stream_handle(stream0),
                                    _stream_handle(stream1)))
        self._h = handle

    def close(self) -> int:
        """Destroys the context; returns iso_destroy's status (ISO_ERR_HIP if the last pass was invalid)."""
        rc = ISO_OK
        if getattr(self, "_h", None):
            rc = self._lib.iso_destroy(self._h)
            self._h = None
        return rc

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    # ---- entry points (same names as the C ABI, without the prefix) ----------------------------
    def sync(self) -> None:
        _check(self._lib.iso_sync(self._h))

    def quantize_rows_fp8(self, x, rows: int, cols: int, q, scale, stream=None) -> None:
        _check(self._lib.iso_quantize_rows_fp8(self._h, _ptr(x), rows, cols, _ptr(q), _ptr(scale), _stream_handle(stream)))

    def rmsnorm_fp8(self, x, delta, g, q, scale, T: int, stream=None) -> None:
        _check(self._lib.iso_rmsnorm_fp8(self._h, _ptr(x), _ptr(delta) if delta is not None else None, _ptr(g), _ptr(q),
                                         _ptr(scale), T, _stream_handle(stream)))

    def gemm_fp8(self, a8, sa, w8, sw, c, M: int, N: int, K: int, stream=None) -> None:
        _check(self._lib.iso_gemm_fp8(self._h, _ptr(a8), _ptr(sa), _ptr(w8), _ptr(sw), _ptr(c), M, N, K,
                                      _stream_handle(stream)))

    def add_fp8_weights(self, w: Dict[str, "DeviceArray"]) -> Dict[str, "DeviceArray"]:
        """Quantises the four matrices of an uploaded bf16 layer per output row and returns the layer with the
        FP8 copies and their scales added (what ISO_FLAG_FP8_GEMM reads)."""
        out = dict(w)
        for name, sname in (("w_qkv", "s_qkv"), ("w_o", "s_o"), ("w_gate_up", "s_gate_up"), ("w_down", "s_down")):
            rows, cols = w[name].shape
            q = DeviceArray((rows, cols), "u8")
            sc = DeviceArray((rows,), "f32")
            self.quantize_rows_fp8(w[name], rows, cols, q, sc, self.stream0)
            out[name + "_f8"], out[sname] = q, sc
        self.sync()
        return out

    def set_gemm_segments(self, n: int) -> None:
        _check(self._lib.iso_set_gemm_segments(self._h, n))

    def set_flags(self, flags: int) -> None:
        _check(self._lib.iso_set_flags(self._h, flags))

    def timing_enable(self, on: bool) -> None:
        _check(self._lib.iso_timing_enable(self._h, 1 if on else 0))

    def timing_read(self) -> Dict[str, tuple]:
        """{kind: (total_ms, launches)} for every kernel kind recorded since timing_enable(True)."""
        out = {}
        for i, name in enumerate(KERNEL_KINDS):
            ms, n = ctypes.c_double(), ctypes.c_int()
            _check(self._lib.iso_timing_read(self._h, i, ctypes.byref(ms), ctypes.byref(n)))
            out[name] = (ms.value, n.value)
        return out

    def host_sink(self) -> int:
        return self._lib.iso_host_sink(self._h)

    def layer_prefill(self, w: Dict[str, object], x, k_cache, v_cache, T: int, split: int,
                      comm: int = ISO_COMM_NONE, sched: int = ISO_SCHED_OVERLAP) -> None:
        ws = pack_weights(w)
        _check(self._lib.iso_layer_prefill(self._h, ctypes.byref(ws), _ptr(x), _ptr(k_cache), _ptr(v_cache),
                                           T, split, comm, sched))

    def stack_prefill(self, layers: Sequence[Dict[str, object]], x, k_caches, v_caches, T: int, split: int,
                      comm: int = ISO_COMM_NONE, sched: int = ISO_SCHED_OVERLAP) -> None:
        arr = (IsoWeights * len(layers))(*[pack_weights(w) for w in layers])
        _check(self._lib.iso_stack_prefill(self._h, arr, len(layers), _ptr(x), _ptr(k_caches), _ptr(v_caches),
                                           T, split, comm, sched))

    def stack_prefill_chunks(self, layers: Sequence[Dict[str, object]], x, k_caches, v_caches, T: int,
                             bounds: Sequence[int], comm: int = ISO_COMM_NONE,
                             sched: int = ISO_SCHED_OVERLAP) -> None:
        """bounds: the ascending cut points; len(bounds) + 1 chunks."""
        arr = (IsoWeights * len(layers))(*[pack_weights(w) for w in layers])
        cuts = (ctypes.c_int * max(1, len(bounds)))(*[int(b) for b in bounds])
        _check(self._lib.iso_stack_prefill_chunks(self._h, arr, len(layers), _ptr(x), _ptr(k_caches), _ptr(v_caches),
                                                  T, cuts if len(bounds) else None, len(bounds) + 1, comm, sched))

    def attn_chunk(self, q, k_cache, v_cache, out, Tc: int, q_offset: int, kv_len: int, stream=None) -> None:
        _check(self._lib.iso_attn_chunk(self._h, _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(out), Tc, q_offset,
                                        kv_len, _stream_handle(stream)))

    def gemm_rowpar(self, a, w, c, M: int, N: int, K: int, stream=None, host_sink: Optional[int] = None) -> None:
        _check(self._lib.iso_gemm_rowpar(self._h, _ptr(a), _ptr(w), _ptr(c), M, N, K, _stream_handle(stream),
                                         host_sink))

    def gemm_rowpar_static(self, a, w, c, M: int, N: int, K: int, stream=None) -> None:
        _check(self._lib.iso_gemm_rowpar_static(self._h, _ptr(a), _ptr(w), _ptr(c), M, N, K, _stream_handle(stream)))

    def streamk_status_word(self):
        """ctypes pointer to the pinned status word of the stream-K GEMM (None for an fp32 context)."""
        p = self._lib.iso_streamk_status_word(self._h)
        return p if p else None

    def rmsnorm(self, x, g, y, T: int, stream=None) -> None:
        _check(self._lib.iso_rmsnorm(self._h, _ptr(x), _ptr(g), _ptr(y), T, _stream_handle(stream)))

    def residual_rmsnorm(self, x, delta, g, y, T: int, stream=None) -> None:
        _check(self._lib.iso_residual_rmsnorm(self._h, _ptr(x), _ptr(delta), _ptr(g), _ptr(y), T,
                                              _stream_handle(stream)))

    def rope_kv_write(self, qkv, k_cache, v_cache, Tc: int, q_offset: int, stream=None) -> None:
        _check(self._lib.iso_rope_kv_write(self._h, _ptr(qkv), _ptr(k_cache), _ptr(v_cache), Tc, q_offset,
                                           _stream_handle(stream)))

    def swiglu(self, gu, a, T: int, stream=None) -> None:
        _check(self._lib.iso_swiglu(self._h, _ptr(gu), _ptr(a), T, _stream_handle(stream)))
