"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (library
defaults).  Where the oracle cannot replay the whole buffer in seconds, sampled windows (plus the
windows around every ring-chunk boundary) are folded by the oracle one by one; properties that hold
at any size (all ranks identical) are checked on the whole buffer on the GPU side."""
import numpy as np
import pytest

import workload_inputs as wi
from oracle import ring_data as rd

pytestmark = pytest.mark.gpu


def _windows(n, R, eb, rng, nwin=48, width=2048):
    ce = rd.chunk_elems(n, R, eb)
    wins = []
    for c in range(1, R):                       # straddle every chunk boundary
        lo = max(0, c * ce - width // 2)
        wins.append((lo, min(n, lo + width)))
    wins.append((0, min(n, width)))
    wins.append((max(0, n - width), n))         # the ragged tail
    for _ in range(nwin):
        lo = int(rng.integers(0, max(1, n - width)))
        wins.append((lo, min(n, lo + width)))
    return ce, wins


def test_config2_largest_size_sampled():
    """R = 8, fp32, 256 MiB per rank, N(0,1) drawn on the device from a fixed seed."""
    import torch
    import paper_2303_06324_amd as dfx
    R, n = 8, (256 << 20) // 4
    g = torch.Generator(device="cuda")
    g.manual_seed(1234)
    send = [torch.randn(n, device="cuda", dtype=torch.float32, generator=g) for _ in range(R)]
    recv = [torch.full((n,), float("nan"), device="cuda", dtype=torch.float32) for _ in range(R)]
    torch.cuda.synchronize()
    ctx = dfx.Context(R)
    try:
        ctx.prepare(0, dfx.ALLREDUCE, n, dfx.F32)
        for it in range(2):                      # second invocation reuses connectors mid-ring
            for r in range(R):
                assert ctx.submit(r, 0, send[r].data_ptr(), recv[r].data_ptr()) == dfx.OK
            assert ctx.wait_all(30.0) == dfx.OK
        ctx.stop()
    finally:
        ctx.finalize()
    for r in range(1, R):                        # every rank ends with identical bits
        assert torch.equal(recv[0].view(torch.int32), recv[r].view(torch.int32))
    rng = np.random.default_rng(7)
    ce, wins = _windows(n, R, 4, rng)
    assert ce == n // 8                          # "chunk = size/8"
    for lo, hi in wins:
        blocks = [s[lo:hi].cpu().numpy() for s in send]
        got = recv[3][lo:hi].cpu().numpy()
        want = np.empty(hi - lo, np.float32)
        i = lo
        while i < hi:                            # a window may straddle a chunk boundary
            c = i // ce
            j = min(hi, (c + 1) * ce)
            want[i - lo:j - lo] = rd.fold_rotated([b[i - lo:j - lo] for b in blocks], c + 1, rd.F32)
            i = j
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), (lo, hi)
        ref = rd.sum_f64(blocks, rd.F32)
        assert np.all(np.abs(got.astype(np.float64) - ref) <= 1e-6 * rd.abs_sum_f64(blocks, rd.F32))


def test_other_kinds_at_the_largest_size():
    """All-gather, reduce-scatter, broadcast and reduce at 256 MiB of largest per-rank buffer, fp32, library
    defaults (the configuration of the bench's table of kinds: direct steps, several slices per channel share,
    512 KiB / 64 KiB slices for the chains).  All-gather and broadcast are compared whole, on the device, with
    their definitions (concatenation / the root's buffer); the reducing kinds on sampled windows that the oracle
    folds one by one; buffers a kind must not write keep their fill pattern."""
    import torch
    import paper_2303_06324_amd as dfx
    R, n, root = 8, (256 << 20) // 4, 3
    blk = n // R
    g = torch.Generator(device="cuda")
    g.manual_seed(4321)
    send = [torch.randn(n, device="cuda", dtype=torch.float32, generator=g) for _ in range(R)]
    recv = [torch.empty(n, device="cuda", dtype=torch.float32) for _ in range(R)]
    rng = np.random.default_rng(11)

    def run(ctx, cid):
        for t in recv:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        for r in reversed(range(R)):
            assert ctx.submit(r, cid, send[r].data_ptr(), recv[r].data_ptr()) == dfx.OK
        assert ctx.wait_all(30.0) == dfx.OK

    def windows(length, nwin=24, width=4096):
        wins = [(0, width), (length - width, length)]
        wins += [(lo, lo + width) for lo in map(int, rng.integers(0, length - width, size=nwin))]
        return wins

    ctx = dfx.Context(R)
    try:
        ctx.prepare(0, dfx.ALLGATHER, blk, dfx.F32)
        ctx.prepare(1, dfx.REDUCESCATTER, blk, dfx.F32)
        ctx.prepare(2, dfx.BROADCAST, n, dfx.F32, dfx.SUM, root)
        ctx.prepare(3, dfx.REDUCE, n, dfx.F32, dfx.SUM, root)
        assert ctx.coll_info(0)["rounds"] == 4 and ctx.coll_info(0)["nprim"] == R + 1
        assert ctx.coll_info(1)["rounds"] == 4 and ctx.coll_info(1)["nprim"] == R + 1

        run(ctx, 0)                                  # all-gather: every rank ends with the concatenation
        want = torch.cat([s[:blk] for s in send])
        for r in range(R):
            assert torch.equal(recv[r].view(torch.int32), want.view(torch.int32)), r
        del want

        run(ctx, 2)                                  # broadcast: every rank ends with the root's buffer
        for r in range(R):
            assert torch.equal(recv[r].view(torch.int32), send[root].view(torch.int32)), r

        run(ctx, 1)                                  # reduce-scatter: rank r ends with block r, folded from rank r+1 on
        for r in range(R):
            assert bool(torch.isnan(recv[r][blk:]).all()), r        # nothing written beyond the block
            for lo, hi in windows(blk, nwin=6):
                blocks = [s[r * blk + lo:r * blk + hi].cpu().numpy() for s in send]
                got = recv[r][lo:hi].cpu().numpy()
                want_w = rd.fold_rotated(blocks, r + 1, rd.F32)
                assert np.array_equal(got.view(np.uint32), want_w.view(np.uint32)), (r, lo, hi)

        run(ctx, 3)                                  # reduce: the root ends with the fold along the chain root+1 .. root
        for r in range(R):
            if r != root:
                assert bool(torch.isnan(recv[r]).all()), r
        for lo, hi in windows(n):
            blocks = [s[lo:hi].cpu().numpy() for s in send]
            got = recv[root][lo:hi].cpu().numpy()
            assert np.array_equal(got.view(np.uint32), rd.reduce_fold(blocks, root, rd.F32).view(np.uint32)), (lo, hi)
        ctx.stop()
    finally:
        ctx.finalize()


def test_config3_full_bf16_buckets_random_orders():
    """16 bf16 buckets of 25 MiB, every rank submitting in its own random order."""
    from tests import gpu_harness as gh
    w = wi.config3()
    assert len(w.colls) == 16 and w.colls[0].count == 25 * (1 << 20) // 2
    dw, stats, _ = gh.run_workload(w, gh.make_config(), timeout_s=90.0)
    rng = np.random.default_rng(3)
    for ci in range(16):
        got = dw.results(ci)
        for r in range(1, 8):
            assert np.array_equal(got[0], got[r])
        n = w.colls[ci].count
        ce, wins = _windows(n, 8, 2, rng, nwin=8)
        for lo, hi in wins:
            i = lo
            while i < hi:
                c = i // ce
                j = min(hi, (c + 1) * ce)
                want = rd.fold_rotated([s[i:j] for s in dw.send_host[ci]], c + 1, rd.BF16)
                assert np.array_equal(got[5][i:j], want), (ci, i, j)
                i = j
    assert sum(s["cqe_posted"] for s in stats) == 16 * 8


def test_config4_full_mixed_collectives():
    """64 mixed collectives (4 kinds, 3 dtypes, 4 KiB - 64 MiB), random orders, staggered submits."""
    from tests import gpu_harness as gh
    w = wi.config4()
    assert len(w.colls) == 64
    dw, stats, _ = gh.run_workload(w, gh.make_config(), mode="threads", timeout_s=120.0)
    for ci, c in enumerate(w.colls):
        got = dw.results(ci)
        nbytes = c.send_elems(8) * wi.ELEM_BYTES[c.dtype]
        if nbytes <= (8 << 20):
            want = rd.run_closed_form(c.kind, dw.send_host[ci], c.dtype, c.root, c.op)
            for r in range(8):
                assert np.array_equal(got[r].view(np.uint8), want[r].view(np.uint8)), (ci, r)
        else:                                    # large ones: closed form on rank 0 and one other, identity across ranks
            want = rd.run_closed_form(c.kind, dw.send_host[ci], c.dtype, c.root, c.op)
            for r in (0, 6):
                assert np.array_equal(got[r].view(np.uint8), want[r].view(np.uint8)), (ci, r)
            if c.kind != wi.RS:
                for r in range(1, 8):
                    assert np.array_equal(got[0].view(np.uint8), got[r].view(np.uint8))
    assert sum(s["cqe_posted"] for s in stats) == 64 * 8


def test_config5_full_1024_small_allreduces():
    from tests import gpu_harness as gh
    w = wi.config5()
    assert len(w.colls) == 1024
    dw, stats, _ = gh.run_workload(w, gh.make_config(), mode="threads", timeout_s=120.0)
    for ci in range(0, 1024):
        c = w.colls[ci]
        want = rd.all_reduce_fold(dw.send_host[ci], c.dtype)
        got = dw.results(ci)
        for r in (0, 7) if ci % 16 else range(8):
            assert np.array_equal(got[r].view(np.uint8), want.view(np.uint8)), (ci, r)
    assert sum(s["cqe_posted"] for s in stats) == 1024 * 8
    assert max(s["max_taskq"] for s in stats) <= 1024


def test_allreduce_beyond_4GiB_offsets_sampled():
    """R = 2, int32, 5 GiB + a ragged tail per rank: byte offsets inside one buffer pass 2^32, thousands of
    slices per channel.  Integer sums are exact in any order, so whole-buffer checks run on the device too;
    sampled windows (chunk boundary, both ends, around the 4 GiB mark, random) go through the oracle."""
    import torch
    import paper_2303_06324_amd as dfx
    R, n = 2, (5 << 30) // 4 + 12345
    g = torch.Generator(device="cuda")
    g.manual_seed(99)
    send = [torch.randint(-(1 << 20), 1 << 20, (n,), device="cuda", dtype=torch.int32, generator=g) for _ in range(R)]
    recv = [torch.full((n,), -7, device="cuda", dtype=torch.int32) for _ in range(R)]
    torch.cuda.synchronize()
    ctx = dfx.Context(R)
    try:
        ctx.prepare(0, dfx.ALLREDUCE, n, dfx.I32)
        info = ctx.coll_info(0)
        assert info["rounds"] > 100
        for r in range(R):
            assert ctx.submit(r, 0, send[r].data_ptr(), recv[r].data_ptr()) == dfx.OK
        assert ctx.wait_all(60.0) == dfx.OK
        ctx.stop()
    finally:
        ctx.finalize()
    assert torch.equal(recv[0], recv[1])
    assert torch.equal(recv[0], send[0] + send[1])           # exact, order-free; on the device
    rng = np.random.default_rng(8)
    ce, wins = _windows(n, R, 4, rng, nwin=24)
    mark = (4 << 30) // 4
    wins.append((mark - 1024, mark + 1024))
    for lo, hi in wins:
        blocks = [s[lo:hi].cpu().numpy() for s in send]
        got = recv[1][lo:hi].cpu().numpy()
        want = np.empty(hi - lo, np.int32)
        i = lo
        while i < hi:
            c = i // ce
            j = min(hi, (c + 1) * ce)
            want[i - lo:j - lo] = rd.fold_rotated([b[i - lo:j - lo] for b in blocks], c + 1, rd.I32)
            i = j
        assert np.array_equal(got, want), (lo, hi)
