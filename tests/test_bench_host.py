"""Host-side checks of bench.py that need no GPU: the byte counts behind the roofline figures against the
primitive programs of the scheduling model, and the refusal of more than one GPU."""
import os
import subprocess
import sys

import pytest

import bench
from oracle import sched_model as sm

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

# blocks read / written by one primitive (send buffer, recv buffer, connector slot, or the previous rank's
# buffer in place of a slot); the primitive table of Sec. 4.2 and the direct variants of it
IO = {
    "send": (1, 1), "copy_send": (1, 2), "copy": (1, 1),
    "recv_reduce_send": (2, 1), "recv_reduce_copy_send": (2, 2), "recv_reduce_copy": (2, 1),
    "recv_copy_send": (1, 2), "recv_copy": (1, 1),
    "notify": (0, 0), "drain": (0, 0), "copy_notify": (1, 1),
    "direct_reduce_send": (2, 1), "direct_reduce_copy_notify": (2, 1), "direct_reduce_copy": (2, 1),
    "recv_reduce_copy_notify": (2, 1), "direct_copy_notify": (1, 1), "direct_copy": (1, 1),
    # fold steps (R ranks): chunk r out of all R send buffers into the own recv buffer (reduce-scatter) or into
    # all R recv buffers (all-reduce)
    "fold_all": lambda R: (R, 1), "fold_scatter": lambda R: (R, R), "last_wait": (0, 0),
    "fold_root": lambda R: (R, 1), "gather_pub": lambda R: (R, R), "last_wait_red": (0, 0),
}


def _blocks_moved(kind, R, direct, root=0, fold=False):
    blocks = [(8 * j, 8 * j + 8) for j in range(R)]
    total = 0
    for r in range(R):
        for name, _, _ in sm.program(kind, R, r, root, blocks, blocks, direct, fold):
            assert set(IO) == set(sm.PRIMS), "every primitive of the model is priced here"
            io = IO[name]
            total += sum(io(R) if callable(io) else io)
    return total


@pytest.mark.parametrize("R", [2, 3, 8, 16])
def test_roofline_byte_counts_follow_from_the_primitive_programs(R):
    """The algorithmic bytes of an all-reduce, (6R-4) x M by the primitive table and (5R-5) x M with the
    direct steps, are the sums over the per-rank programs of what each primitive reads and writes
    (a chunk is M/R); likewise the figures of the other kinds in the kinds table."""
    M = R << 16
    chunk = M // R
    assert _blocks_moved(sm.AR, R, False) * chunk == bench.algorithmic_bytes(M, R)
    assert _blocks_moved(sm.AR, R, True) * chunk == bench.moved_bytes(M, R)
    assert _blocks_moved(sm.AR, R, False, fold=True) * chunk == bench.fold_bytes(M, R)      # 2R x M in fold steps
    # per rank, in blocks: all-gather 3R-1 -> 2R, reduce-scatter 3R-1 -> 3R-3; chains, in messages: broadcast
    # 3R-1 -> 2R, reduce 3R-1 -> 3R-3
    assert _blocks_moved(sm.AG, R, False) == R * (3 * R - 1) and _blocks_moved(sm.AG, R, True) == R * 2 * R
    assert _blocks_moved(sm.RS, R, False) == R * (3 * R - 1) and _blocks_moved(sm.RS, R, True) == R * (3 * R - 3)
    assert _blocks_moved(sm.BC, R, False, root=1) == 3 * R - 1 and _blocks_moved(sm.BC, R, True, root=1) == 2 * R
    assert _blocks_moved(sm.RD, R, False, root=1) == 3 * R - 1 and _blocks_moved(sm.RD, R, True, root=1) == 3 * R - 3


def test_measured_traffic_constant_is_the_moved_bytes_of_the_headline_workload():
    """The counter-measured HBM traffic that bench.py reports for the 256 MiB workload lies within 0.2 % of
    what the direct steps have to move."""
    want = bench.moved_bytes(256 << 20, 8)
    assert abs(bench.MEASURED_TRAFFIC_BYTES - want) / want < 2e-3


def test_more_than_one_gpu_is_refused():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in res.stderr and res.stdout.strip() == ""
