"""The kernel's index arithmetic, walked on the CPU (dfx_check_geometry compiles the same functions as the
kernel: workgroup -> (rank, channel), connector addresses, primitive sequences, slice geometry, the order of
slices and primitives).  No GPU: for every workgroup of the grid, every address the kernel would form is
checked against the buffers and the connector block, the writes to each recv buffer must tile it exactly,
and both ends of every connector must agree.

It covers the workload of the run that once ended in a GPU memory fault (every kind at 256 MiB and
all-reduces of 8 KiB - 64 MiB, under a third workgroup labelling that has since been taken out of the
kernel): that labelling, wg_map 2 here, is checked along with the two the kernel offers."""
import itertools

import pytest

import paper_2303_06324_amd as dfx

KINDS = [dfx.ALLREDUCE, dfx.ALLGATHER, dfx.REDUCESCATTER, dfx.BROADCAST, dfx.REDUCE]


def _cfg(**kw):
    cfg = dfx.config_default()
    for k, v in kw.items():
        setattr(cfg, k, v)
    return cfg


@pytest.mark.parametrize("wg_map", [0, 1, 2])
def test_workload_of_the_faulting_run_under_every_map(wg_map):
    R, n = 8, (256 << 20) // 4
    cases = [(dfx.ALLREDUCE, n), (dfx.ALLGATHER, n // R), (dfx.REDUCESCATTER, n // R), (dfx.BROADCAST, n), (dfx.REDUCE, n),
             (dfx.ALLREDUCE, 2048), (dfx.ALLREDUCE, 1 << 18), (dfx.ALLREDUCE, 1 << 21), (dfx.ALLREDUCE, 1 << 24),
             (dfx.BROADCAST, 1 << 21)]
    for i, (kind, count) in enumerate(cases):                       # coll ids 0 .. 9 as in that run
        assert dfx.check_geometry(R, kind, count, dfx.F32, root=3, coll_id=i, wg_map=wg_map) == "", (kind, count)
    for p in range(13, 27):                                         # the all-reduce size sweep
        assert dfx.check_geometry(R, dfx.ALLREDUCE, (1 << p) // 4, dfx.F32, wg_map=wg_map) == ""
    n3 = 25 * (1 << 20) // 2                                        # the sixteen bf16 buckets
    for i in range(16):
        assert dfx.check_geometry(R, dfx.ALLREDUCE, n3, dfx.BF16, coll_id=i, wg_map=wg_map) == ""


@pytest.mark.parametrize("kind", KINDS)
def test_ragged_counts_rank_counts_and_dtypes(kind):
    for R, count, dtype in itertools.product([1, 2, 3, 5, 8, 16], [0, 1, 7, 4099, 100003, (1 << 20) + 24], [dfx.F32, dfx.BF16]):
        cfg = _cfg(max_channels=min(32, 256 // R))
        for root in {0, R - 1}:
            for wg_map in (0, 1):
                msg = dfx.check_geometry(R, kind, count, dtype, root=root, coll_id=count % 7, wg_map=wg_map, cfg=cfg)
                assert msg == "", (kind, R, count, dtype, root, wg_map, msg)


@pytest.mark.parametrize("knobs", [dict(direct=0), dict(direct_min_bytes=0), dict(window=1), dict(window=4, nslots=8), dict(nslots=2),
                                   dict(slot_bytes=4096, max_channels=4), dict(chan_spread=0), dict(chan_min_bytes=1 << 20),
                                   dict(direct_min_bytes=0, slot_bytes=16 << 10, max_channels=2, window=1),
                                   dict(fold_slice_bytes=4096), dict(fold_slice_bytes=48, max_channels=2), dict(order_policy=1, fold_slice_bytes=32 << 10),
                                   dict(fold_slice_bytes=1 << 16, fold_max_bytes=1 << 30)])
def test_scheduler_knobs(knobs):
    cfg = _cfg(**knobs)
    for kind in KINDS:
        for count in (8, 30008, (3 << 20) + 8, 1 << 24):
            for cid in (0, 5, 1023):
                msg = dfx.check_geometry(8, kind, count, dfx.F16, op=dfx.MAX, root=5, coll_id=cid, cfg=cfg)
                assert msg == "", (knobs, kind, count, cid, msg)


def test_a_large_offset_case():
    """5 GiB + a ragged tail per rank on two ranks: byte offsets beyond 2^32, thousands of slices per channel."""
    assert dfx.check_geometry(2, dfx.ALLREDUCE, (5 << 30) // 4 + 12345, dfx.I32) == ""


def test_it_refuses_what_it_cannot_check():
    assert dfx.check_geometry(8, dfx.BROADCAST, 1024, dfx.F32, root=9) != ""
    assert dfx.check_geometry(8, dfx.ALLREDUCE, 1024, dfx.F32, wg_map=3) != ""
