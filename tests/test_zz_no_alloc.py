"""The entry point that allocates nothing (dfx_collective_noalloc: the daemon kernel on the library's static
scratch array) against the context path (dfx_init + dfx_prepare + dfx_submit_all) on the same inputs, bit for
bit, and against the oracle: two calls in a row, the second with a smaller input, then the other kinds."""
import numpy as np
import pytest

import workload_inputs as wi
from oracle import ring_data as rd

pytestmark = pytest.mark.gpu


def _both_paths(kind, dtype, count, R, root=0, op=wi.SUM, seed=0):
    import torch
    import paper_2303_06324_amd as dfx
    from paper_2303_06324_amd import harness as gh
    w = wi.Workload(f"noalloc_{kind}_{dtype}_{count}", R, [wi.CollSpec(0, kind, dtype, count, root, op)], [[0]] * R,
                    seed=seed, cfg=88)
    # the context path (the existing entry points)
    dw_ctx = gh.DeviceWorkload(w)
    gh.run_workload(w, gh.make_config(max_channels=min(32, 256 // R)), dw=dw_ctx, timeout_s=30.0)
    # the entry point that allocates nothing, on buffers of its own
    dw = gh.DeviceWorkload(w)
    status = torch.full((1,), 0xdead, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    rc = dfx.collective_noalloc(R, kind, count, dtype, op, root, [t.data_ptr() for t in dw.send[0]],
                                [t.data_ptr() for t in dw.recv[0]], status.data_ptr(), None)
    assert rc == dfx.OK, dfx.strerror(rc)
    torch.cuda.synchronize()
    assert int(status.item()) == 0, hex(int(status.item()))
    want = rd.run_closed_form(kind, dw.send_host[0], dtype, root, op)
    a, b = dw_ctx.results(0), dw.results(0)
    for r in range(R):
        assert np.array_equal(a[r].view(np.uint8), b[r].view(np.uint8)), (kind, dtype, count, r)
        if kind == wi.RD and r != root:
            assert np.all(b[r].view(np.uint8) == 0xA5)
        else:
            assert np.array_equal(b[r].view(np.uint8), want[r].view(np.uint8)), (kind, dtype, count, r)
    dw.check_untouched()


def test_noalloc_two_calls_in_a_row_second_one_smaller():
    _both_paths(wi.AR, wi.F32, 17 * (1 << 20) + 7, 8, seed=1)    # 68 MiB per rank: the ring, direct steps, many slices through the scratch's slots
    _both_paths(wi.AR, wi.F32, 4099, 8, seed=2)                   # smaller: one channel, fold steps
    _both_paths(wi.AR, wi.BF16, 300007, 8, op=wi.MAX, seed=3)


@pytest.mark.parametrize("kind,dtype,count,R,root", [(wi.AG, wi.F16, 40008, 8, 0), (wi.RS, wi.I32, 30001, 5, 0), (wi.RS, wi.F32, 1 << 20, 8, 0),
                                                     (wi.BC, wi.F32, 1 << 20, 8, 3), (wi.RD, wi.BF16, 270001, 3, 2),
                                                     (wi.AR, wi.F32, 1, 16, 0), (wi.AR, wi.I32, 0, 4, 0)])
def test_noalloc_other_kinds_and_rank_counts(kind, dtype, count, R, root):
    _both_paths(kind, dtype, count, R, root=root, seed=count % 97)


def test_noalloc_rejects_what_it_cannot_hold():
    import torch
    import paper_2303_06324_amd as dfx
    from paper_2303_06324_amd import harness as gh
    buf = torch.zeros(64, dtype=torch.uint8, device="cuda")
    p = [buf.data_ptr()] * 8
    too_many = dfx.NOALLOC_MAX_BYTES // 4 + 1
    assert dfx.collective_noalloc(8, dfx.ALLREDUCE, too_many, dfx.F32, dfx.SUM, 0, p, p) == dfx.ERR_TOO_LARGE
    assert dfx.collective_noalloc(8, dfx.ALLGATHER, too_many // 8 + 1, dfx.F32, dfx.SUM, 0, p, p) == dfx.ERR_TOO_LARGE
    q = [buf.data_ptr()] * 65
    assert dfx.collective_noalloc(65, dfx.ALLREDUCE, 16, dfx.F32, dfx.SUM, 0, q, q) == dfx.ERR_INVALID_ARG
    assert dfx.collective_noalloc(8, dfx.BROADCAST, 16, dfx.F32, dfx.SUM, 8, p, p) == dfx.ERR_INVALID_ARG
    # refused while a context's daemon is resident on the device
    ctx = dfx.Context(2, gh.make_config(quit_idle_us=0, max_channels=4))
    try:
        assert ctx.start() == dfx.OK
        assert dfx.collective_noalloc(2, dfx.ALLREDUCE, 16, dfx.F32, dfx.SUM, 0, p[:2], p[:2]) == dfx.ERR_BUSY
        assert ctx.stop() == dfx.OK
    finally:
        ctx.finalize()
