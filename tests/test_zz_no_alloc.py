"""The entry point that allocates nothing (iso_gemm_rowpar_static: stream-K GEMM whose workspace is a static device
array) against the existing iso_gemm_rowpar and the oracle, through the C ABI: two calls in a row, the second with a
smaller input, so that what the first call left in the shared array (raised flags, partial tiles) must not leak into
the second."""
import numpy as np
import pytest

import paper_2409_11155_amd as iso      # first: binds libiso to the HIP runtime it was built against
import iso_inputs
from oracle import iso_oracle as orc

pytestmark = pytest.mark.gpu

TOL_STEP_BF16 = 1e-2       # single bf16 step: output rounding 2^-8, fp32 accumulation
NAN_BYTE = 0xFF


def h64(a):
    return iso_inputs.to_f64(a, "bf16")


def test_static_workspace_gemm_two_calls_in_a_row_second_one_smaller():
    dt = "bf16"
    # the first product spreads every tile column over several workgroups (partial tiles and flags in use), the
    # second is smaller in all three sizes, has a ragged last tile, and uses fewer workgroups' worth of k-slices
    cases = [(1024, 2304, 4096), (300, 520, 1024)]
    with iso.Context(iso.make_cfg(256, 4, 4, 64, 64, dt, 256)) as ctx:
        ops = []
        for i, (M, N, K) in enumerate(cases):
            a = iso_inputs.randn((M, K), seed=300 + i, dtype=dt)
            w = iso_inputs.randn((N, K), seed=400 + i, dtype=dt, scale=K ** -0.5)
            ops.append((a, w, iso.DeviceArray.from_numpy(a, dt), iso.DeviceArray.from_numpy(w, dt),
                        iso.DeviceArray((M, N), dt, fill_byte=NAN_BYTE)))
        # both calls back to back in one stream, nothing in between
        for (M, N, K), (_, _, ad, wd, cd) in zip(cases, ops):
            ctx.gemm_rowpar_static(ad, wd, cd, M, N, K, ctx.stream0)
        ctx.sync()
        for (M, N, K), (a, w, ad, wd, cd) in zip(cases, ops):
            got = cd.numpy()
            ref = orc.linear(h64(a), h64(w))
            err = orc.max_rel_err(h64(got), ref)
            assert err <= TOL_STEP_BF16, (M, N, K, err)
            # the existing entry point, by its own launch rule and forced through its stream-K launch
            for flags in (0, 6 << 8):
                ctx.set_flags(flags)
                c2 = iso.DeviceArray((M, N), dt, fill_byte=NAN_BYTE)
                ctx.gemm_rowpar(ad, wd, c2, M, N, K, ctx.stream0)
                ctx.sync()
                other = c2.numpy()
                assert orc.max_rel_err(h64(other), ref) <= TOL_STEP_BF16
                # two bf16 roundings of sums taken in different orders: within twice the step bound of each other
                assert orc.max_rel_err(h64(got), h64(other)) <= 2 * TOL_STEP_BF16, (M, N, K, flags)
                if flags == 6 << 8:
                    # same kernel, same launch shape, same order of the partial sums: the same bits
                    np.testing.assert_array_equal(got, other)
            ctx.set_flags(0)


def test_static_workspace_gemm_rejects_what_it_cannot_take():
    with iso.Context(iso.make_cfg(256, 4, 4, 64, 64, "bf16", 64)) as ctx:
        t = iso.DeviceArray((64, 64), "bf16", fill_byte=0)
        for (M, N, K), code in (((64, 64, 72), iso.ISO_ERR_SHAPE),      # K not a multiple of 64
                                ((64, 60, 64), iso.ISO_ERR_SHAPE),      # N not a multiple of 8
                                ((0, 64, 64), iso.ISO_ERR_SHAPE),
                                ((1 << 20, 64, 4096), iso.ISO_ERR_SHAPE)):   # M*K beyond 2^31 elements
            with pytest.raises(iso.IsoError) as ei:
                ctx.gemm_rowpar_static(t, t, t, M, N, K, ctx.stream0)
            assert ei.value.code == code, (M, N, K)
    with iso.Context(iso.make_cfg(256, 4, 4, 64, 64, "f32", 64)) as c32:
        t = iso.DeviceArray((64, 64), "f32", fill_byte=0)
        with pytest.raises(iso.IsoError) as ei:
            c32.gemm_rowpar_static(t, t, t, 64, 64, 64, c32.stream0)
        assert ei.value.code == iso.ISO_ERR_DTYPE


def test_static_workspace_gemm_recorded_into_a_graph_and_replayed():
    """What the entry point is for: a caller that records its work into a HIP graph.  The call is captured once (two
    kernel nodes, no memset node, no allocation) and replayed with changing contents of `a`, with eager work and a
    synchronisation between the replays; every replay must give the bits of the eager call on the same operands."""
    from test_gpu_graph import Captured, hip_runtime
    rt = hip_runtime()
    dt, (M, N, K) = "bf16", (1024, 2304, 4096)
    w = iso_inputs.randn((N, K), seed=71, dtype=dt, scale=K ** -0.5)
    a_sets = [iso_inputs.randn((M, K), seed=72 + i, dtype=dt) for i in range(3)]
    with iso.Context(iso.make_cfg(256, 4, 4, 64, 64, dt, 256)) as ctx:
        wd = iso.DeviceArray.from_numpy(w, dt)
        ad = iso.DeviceArray.from_numpy(a_sets[0], dt)
        cd = iso.DeviceArray((M, N), dt, fill_byte=NAN_BYTE)
        eager = iso.DeviceArray((M, N), dt, fill_byte=NAN_BYTE)
        ctx.gemm_rowpar_static(ad, wd, cd, M, N, K, ctx.stream0)          # once eagerly, as for every captured call
        ctx.sync()
        g = Captured(rt, ctx.stream0.handle, lambda: ctx.gemm_rowpar_static(ad, wd, cd, M, N, K, ctx.stream0))
        try:
            for a in a_sets + a_sets[:1]:
                ad.upload(a)                                              # synchronous copy: eager work between replays
                cd.fill(NAN_BYTE)
                ctx.gemm_rowpar_static(ad, wd, eager, M, N, K, ctx.stream0)
                ctx.sync()
                g.launch()
                ctx.sync()
                got = cd.numpy()
                np.testing.assert_array_equal(got, eager.numpy())
                assert orc.max_rel_err(h64(got), orc.linear(h64(a), h64(w))) <= TOL_STEP_BF16
        finally:
            g.destroy()
