"""Entry points recorded into a HIP graph and replayed: every replay must give what the eager call gives.

The graph calls go straight to the HIP runtime that libiso is linked against (the C ABI has no graph functions: a
caller that captures brings its own).  Between replays the test does eager work and synchronises, as a program would.
"""
import ctypes

import numpy as np
import pytest

import paper_2409_11155_amd as iso      # first: binds libiso to the HIP runtime it was built against
import iso_inputs
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

CAPTURE_RELAXED = 2      # hipStreamCaptureModeRelaxed


def hip_runtime():
    """The HIP runtime object already mapped into this process (the one libiso uses)."""
    iso.load()
    with open("/proc/self/maps") as f:
        paths = {line.split()[-1] for line in f if "libamdhip64" in line}
    assert len(paths) == 1, paths
    rt = ctypes.CDLL(paths.pop())
    rt.hipStreamBeginCapture.argtypes = [ctypes.c_void_p, ctypes.c_int]
    rt.hipStreamEndCapture.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_void_p)]
    rt.hipGraphInstantiate.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_char_p,
                                       ctypes.c_size_t]
    rt.hipGraphLaunch.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    rt.hipGraphExecDestroy.argtypes = [ctypes.c_void_p]
    rt.hipGraphDestroy.argtypes = [ctypes.c_void_p]
    return rt


class Captured:
    """Records what `enqueue()` puts on `stream` (and on the streams it forks to) into an executable graph."""

    def __init__(self, rt, stream, enqueue):
        self.rt, self.stream = rt, stream
        assert rt.hipStreamBeginCapture(stream, CAPTURE_RELAXED) == 0
        try:
            enqueue()
        finally:
            graph = ctypes.c_void_p()
            rc = rt.hipStreamEndCapture(stream, ctypes.byref(graph))
        assert rc == 0 and graph.value, rc
        self.graph = graph
        self.exe = ctypes.c_void_p()
        assert rt.hipGraphInstantiate(ctypes.byref(self.exe), graph, None, None, 0) == 0

    def launch(self):
        assert self.rt.hipGraphLaunch(self.exe, self.stream) == 0

    def destroy(self):
        self.rt.hipGraphExecDestroy(self.exe)
        self.rt.hipGraphDestroy(self.graph)


def dev(a, dt):
    return iso.DeviceArray.from_numpy(a, dt)


def test_captured_gemm_of_stream_k_size_replays_correctly():
    """512 x 5120 x 8192 is a shape the eager launch gives to the stream-K kernel (20 k-slices per team on 256
    compute units), whose launches are numbered.  Recorded into a graph the product must take a launch that can be
    replayed: three replays, the output cleared and the same stream-K workspace used by eager launches in between."""
    dt, (M, N, K) = "bf16", (512, 5120, 8192)
    assert iso.gemm_launch_plan(M, N, K, 256)[0] == 6
    a = iso_inputs.randn((M, K), seed=5, dtype=dt)
    w = iso_inputs.randn((N, K), seed=6, dtype=dt, scale=K ** -0.5)
    ref = orc.linear(iso_inputs.to_f64(a, dt), iso_inputs.to_f64(w, dt))
    rt = hip_runtime()
    cfg = iso.make_cfg(256, 4, 4, 64, 64, dt, 256)
    with iso.Context(cfg) as ctx:
        s0 = ctx.stream0.handle
        ad, wd = dev(a, dt), dev(w, dt)
        other = dev(iso_inputs.randn((M, K), seed=7, dtype=dt), dt)      # a different product for the same workspace
        eager = iso.DeviceArray((M, N), dt, fill_byte=0)
        ctx.gemm_rowpar(ad, wd, eager, M, N, K, ctx.stream0)
        ctx.sync()
        assert orc.max_rel_err(iso_inputs.to_f64(eager.numpy(), dt), ref) <= 1e-2
        out = iso.DeviceArray((M, N), dt, fill_byte=0xFF)
        g = Captured(rt, s0, lambda: ctx.gemm_rowpar(ad, wd, out, M, N, K, ctx.stream0))
        ctx.sync()
        first = None
        for rep in range(3):
            out.fill(0xFF)                                             # NaN pattern: a replay must write every element
            ctx.gemm_rowpar(other, wd, eager, M, N, K, ctx.stream0)    # eager stream-K launch between the replays:
                                                                       # other partial tiles, a newer launch number
            g.launch()
            ctx.sync()
            got = out.numpy().copy()
            assert orc.max_rel_err(iso_inputs.to_f64(got, dt), ref) <= 1e-2, rep
            if first is None:
                first = got
            np.testing.assert_array_equal(got, first)
        g.destroy()


def test_captured_iso_layer_replays_bit_identically_to_the_eager_step():
    """A two-chunk ISO step with both transfers (fork to the second stream, K/V event, two copies per chunk, join)
    recorded from stream0 and replayed three times on fresh inputs and NaN-filled caches."""
    dt, d = "bf16", 128
    hidden, nq, nkv, ffn, T, split = 512, 4, 1, 768, 300, 130
    w = iso_inputs.make_layer(hidden, nq, nkv, d, ffn, seed=21, dtype=dt)
    x = iso_inputs.make_hidden(T, hidden, seed=21, dtype=dt)
    sh = orc.LayerShape(hidden, nq, nkv, d, ffn, 1e-6, 10000.0)
    ref = orc.layer_unsplit(iso_inputs.to_f64(x, dt), {k: iso_inputs.to_f64(v, dt) for k, v in w.items()}, sh)["x_out"]
    rt = hip_runtime()
    cfg = iso.make_cfg(hidden, nq, nkv, d, ffn, dt, 320)
    with iso.Context(cfg) as ctx:
        w_dev = iso.upload_weights(w, dt)
        xd = dev(x, dt)
        kc = iso.DeviceArray((320, nkv, d), dt, fill_byte=0xFF)
        vc = iso.DeviceArray((320, nkv, d), dt, fill_byte=0xFF)
        ctx.layer_prefill(w_dev, xd, kc, vc, T, split, iso.ISO_COMM_D2H, iso.ISO_SCHED_OVERLAP)   # eager: also the warm-up
        ctx.sync()
        eager = xd.numpy().copy()
        assert orc.max_rel_err(iso_inputs.to_f64(eager, dt), ref) <= 2e-2
        g = Captured(rt, ctx.stream0.handle,
                     lambda: ctx.layer_prefill(w_dev, xd, kc, vc, T, split, iso.ISO_COMM_D2H, iso.ISO_SCHED_OVERLAP))
        ctx.sync()
        for rep in range(3):
            xd.upload(x)
            kc.fill(0xFF)
            vc.fill(0xFF)
            g.launch()
            ctx.sync()
            np.testing.assert_array_equal(xd.numpy(), eager)
        g.destroy()
