"""Pins for the data oracle (oracle/ring_data.py): everything here runs on the CPU.

Each test checks the oracle against something other than itself: brute force written
element by element, exact integer sums, fp64 error bounds, torch CPU 16-bit arithmetic,
a hand-worked association example, and definitions (concatenation / copy).
"""
import itertools
import os

import numpy as np
import pytest
import torch

import workload_inputs as wi
from oracle import ring_data as rd

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_sends(R, n, dtype, seed=0, sigma=1.0):
    w = wi.Workload("t", R, [wi.CollSpec(0, wi.AR, dtype, n)], [[0]] * R, sigma=sigma, seed=seed, cfg=99)
    return wi.all_sends(w, 0)


# ---------------------------------------------------------------- arithmetic pins
def test_bf16_widen_matches_torch_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ours = rd.bf16_bits_to_f32(bits)
    theirs = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours.view(np.uint32), theirs.view(np.uint32))


def test_bf16_roundtrip_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    f = rd.bf16_bits_to_f32(bits)
    finite_or_inf = ~np.isnan(f)
    back = rd.f32_to_bf16_bits_rne(f)
    assert np.array_equal(back[finite_or_inf], bits[finite_or_inf])
    assert np.all(np.isnan(rd.bf16_bits_to_f32(back[~finite_or_inf])))


def test_bf16_rne_matches_torch_random_and_ties():
    g = np.random.default_rng(1)
    u = g.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    # force many exact ties and near-ties: low half = 0x8000, 0x7fff, 0x8001
    u[:3000:3] = (u[:3000:3] & np.uint32(0xFFFF0000)) | np.uint32(0x8000)
    u[1:3000:3] = (u[1:3000:3] & np.uint32(0xFFFF0000)) | np.uint32(0x7FFF)
    u[2:3000:3] = (u[2:3000:3] & np.uint32(0xFFFF0000)) | np.uint32(0x8001)
    x = u.view(np.float32)
    keep = np.isfinite(x)
    x = x[keep]
    ours = rd.f32_to_bf16_bits_rne(x)
    theirs = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(ours, theirs)


@pytest.mark.parametrize("dtype,tdt", [(rd.BF16, torch.bfloat16), (rd.F16, torch.float16)])
def test_16bit_hop_matches_torch_cpu_add(dtype, tdt):
    g = np.random.default_rng(2)
    n = 1 << 18
    scales = np.exp(g.uniform(-12, 8, size=n)).astype(np.float32)
    a32 = (g.standard_normal(n).astype(np.float32) * scales)
    b32 = (g.standard_normal(n).astype(np.float32) * scales * np.float32(1.0 + 1e-3))
    ta, tb = torch.from_numpy(a32).to(tdt), torch.from_numpy(b32).to(tdt)
    ok = torch.isfinite(ta) & torch.isfinite(tb) & torch.isfinite(ta + tb)
    ta, tb = ta[ok], tb[ok]
    if dtype == rd.BF16:
        a = ta.view(torch.int16).numpy().view(np.uint16)
        b = tb.view(torch.int16).numpy().view(np.uint16)
        want = (ta + tb).view(torch.int16).numpy().view(np.uint16)
    else:
        a, b = ta.numpy(), tb.numpy()
        want = (ta + tb).numpy()
    got = rd.add_hop(a, b, dtype)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


def test_fp16_hop_is_correctly_rounded_vs_fp64():
    # the exact sum of two fp16 values fits in fp64; rounding that once to fp16 is the definition
    g = np.random.default_rng(3)
    a = g.standard_normal(50000).astype(np.float16)
    b = (g.standard_normal(50000) * 3).astype(np.float16)
    want = (a.astype(np.float64) + b.astype(np.float64)).astype(np.float16)
    assert np.array_equal(rd.add_hop(a, b, rd.F16).view(np.uint16), want.view(np.uint16))


def test_int32_hop_wraps():
    a = np.array([2**31 - 1, -2**31, 5, -7], dtype=np.int32)
    b = np.array([1, -1, 6, 7], dtype=np.int32)
    got = rd.add_hop(a, b, rd.I32)
    assert got.tolist() == [-2**31, 2**31 - 1, 11, 0]


def test_fp32_hop_keeps_denormals_and_is_single_add():
    a = np.array([1e-45, 1.0, 3e-39], dtype=np.float32)
    b = np.array([1e-45, 2.0**-24, -1e-39], dtype=np.float32)
    got = rd.add_hop(a, b, rd.F32)
    want = np.array([np.float32(a[i]) + np.float32(b[i]) for i in range(3)], dtype=np.float32)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    assert got[0] != 0.0 and got[2] != 0.0       # gradual underflow, not flushed
    assert got[1] == np.float32(1.0)              # tie to even


# ---------------------------------------------------------------- chunking
@pytest.mark.parametrize("R", range(1, 9))
def test_chunks_partition_message(R):
    for eb in (2, 4):
        for N in range(1, 4 * R + 4):
            cb = rd.chunk_bounds(N, R, eb)
            assert len(cb) == R
            covered = []
            for lo, hi in cb:
                assert 0 <= lo <= hi <= N
                assert (lo * eb) % 16 == 0 or lo == N
                covered.extend(range(lo, hi))
            assert covered == list(range(N))


def test_chunk_is_size_over_R_when_divisible():
    # "chunk = size/8" for the size sweep
    for p in range(13, 29):
        n = (1 << p) // 4
        assert rd.chunk_elems(n, 8, 4) == n // 8


# ---------------------------------------------------------------- all-reduce values
def _brute_allreduce_scalar(sends, dtype):
    """Element-by-element python loop in the rotated rank order; only scalar numpy ops."""
    R, N = len(sends), len(sends[0])
    eb = rd.ELEM_BYTES[dtype]
    per16 = 16 // eb
    ce = -(-(-(-N // R)) // per16) * per16
    out = np.zeros(N, dtype=sends[0].dtype)
    for i in range(N):
        c = i // ce
        order = [(c + 1 + j) % R for j in range(R)]
        if dtype == rd.F32:
            v = np.float32(sends[order[0]][i])
            for r in order[1:]:
                v = np.float32(v + np.float32(sends[r][i]))
        elif dtype == rd.I32:
            v = int(sends[order[0]][i])
            for r in order[1:]:
                v = (v + int(sends[r][i]) + 2**31) % 2**32 - 2**31
        elif dtype == rd.F16:
            v = np.float16(sends[order[0]][i])
            for r in order[1:]:
                v = np.float16(np.float64(v) + np.float64(sends[r][i]))
        else:
            t = torch.tensor([int(np.int16(np.uint16(sends[order[0]][i]).view(np.int16)))],
                             dtype=torch.int16).view(torch.bfloat16)
            for r in order[1:]:
                u = torch.tensor([int(np.uint16(sends[r][i]).view(np.int16))], dtype=torch.int16).view(torch.bfloat16)
                t = t + u
            v = np.uint16(t.view(torch.int16).numpy().view(np.uint16)[0])
        out[i] = v
    return out


@pytest.mark.parametrize("dtype", [rd.F32, rd.BF16, rd.F16, rd.I32])
@pytest.mark.parametrize("R,N", [(1, 5), (2, 9), (3, 12), (4, 37), (8, 64), (8, 131), (5, 3), (8, 7)])
def test_allreduce_replay_fold_bruteforce_agree(dtype, R, N):
    sends = _rand_sends(R, N, dtype, seed=R * 1000 + N)
    rep = rd.all_reduce_replay(sends, dtype)
    fold = rd.all_reduce_fold(sends, dtype)
    brute = _brute_allreduce_scalar(sends, dtype)
    for r in range(R):
        assert np.array_equal(rep[r].view(np.uint8), fold.view(np.uint8)), f"rank {r} differs from closed form"
    assert np.array_equal(fold.view(np.uint8), brute.view(np.uint8))


def test_allreduce_handworked_association():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "ring_fold_handworked.txt")) if l.strip() and l[0] != "#"]
    R, N = 3, 12
    sends = [np.full(N, 2.0**24, np.float32), np.ones(N, np.float32), np.ones(N, np.float32)]
    for impl in (lambda: rd.all_reduce_replay(sends, rd.F32)[0], lambda: rd.all_reduce_fold(sends, rd.F32)):
        out = impl()
        for c, want in rows:
            c = int(c)
            assert np.all(out[4 * c:4 * c + 4] == np.float32(float(want))), (c, out)


@pytest.mark.parametrize("orders", list(itertools.product([(0, 1), (1, 0)], repeat=2)))
def test_config1_values_exact_integers(orders):
    w = wi.config1(*orders)
    for ci in range(2):
        sends = wi.all_sends(w, ci)
        assert all(np.all(s == np.round(s)) and np.all(np.abs(s) <= 8) for s in sends)
        exact = np.sum(np.stack([s.astype(np.int64) for s in sends]), axis=0)
        for out in rd.all_reduce_replay(sends, rd.F32):
            assert np.array_equal(out.astype(np.int64), exact)
            assert np.array_equal(out, exact.astype(np.float32))


@pytest.mark.parametrize("dtype,u", [(rd.F32, 2.0**-24), (rd.F16, 2.0**-11), (rd.BF16, 2.0**-8)])
def test_allreduce_error_bound_vs_fp64(dtype, u):
    R, N = 8, 8 * 4096 + 24
    sigma = 1.0 if dtype != rd.BF16 else 1e-2
    sends = _rand_sends(R, N, dtype, seed=7, sigma=sigma)
    out = rd.to_f64(rd.all_reduce_fold(sends, dtype), dtype)
    ref = rd.sum_f64(sends, dtype)
    bound = (R - 1) * u * (1 + u) ** (R - 1) * rd.abs_sum_f64(sends, dtype)
    tiny = 2.0**-24 if dtype == rd.F16 else 0.0      # fp16 subnormal spacing
    assert np.all(np.abs(out - ref) <= bound + (R - 1) * tiny)


def test_allreduce_R2_is_single_add():
    a, b = _rand_sends(2, 1000, rd.F32, seed=5)
    out = rd.all_reduce_replay([a, b], rd.F32)
    assert np.array_equal(out[0], a + b) and np.array_equal(out[1], b + a)


def test_allreduce_int32_bruteforce_with_overflow():
    g = np.random.default_rng(11)
    R, N = 8, 1003
    sends = [g.integers(-2**31, 2**31, size=N, dtype=np.int64).astype(np.int32) for _ in range(R)]
    want = (np.sum(np.stack([s.astype(np.int64) for s in sends]), axis=0) + 2**31) % 2**32 - 2**31
    for out in rd.all_reduce_replay(sends, rd.I32):
        assert np.array_equal(out.astype(np.int64), want)


def test_planted_association_mistake_is_caught():
    """A fold that starts at rank c instead of c+1 (an off-by-one a reader could make) must
    disagree with the oracle on inputs where association matters: guards the pin's power."""
    R, N = 8, 8 * 64
    sends = _rand_sends(R, N, rd.F32, seed=13)
    good = rd.all_reduce_fold(sends, rd.F32)
    bad = np.zeros_like(good)
    for c, (lo, hi) in enumerate(rd.chunk_bounds(N, R, 4)):
        bad[lo:hi] = rd.fold_rotated([x[lo:hi] for x in sends], c, rd.F32)
    assert not np.array_equal(good, bad)


# ---------------------------------------------------------------- the other collectives
@pytest.mark.parametrize("dtype", [rd.F32, rd.F16, rd.I32, rd.BF16])
@pytest.mark.parametrize("R,count", [(1, 4), (2, 8), (3, 5), (8, 16), (8, 13)])
def test_allgather_is_concatenation(dtype, R, count):
    sends = _rand_sends(R, count, dtype, seed=21)
    want = np.concatenate(sends)
    for out in rd.all_gather_replay(sends, dtype):
        assert np.array_equal(out.view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("dtype", [rd.F32, rd.F16, rd.I32])
@pytest.mark.parametrize("R", [1, 2, 3, 8])
def test_broadcast_is_copy_of_root(dtype, R):
    sends = _rand_sends(R, 77, dtype, seed=22)
    for root in range(R):
        for out in rd.broadcast_replay(sends, root, dtype):
            assert np.array_equal(out.view(np.uint8), sends[root].view(np.uint8))


@pytest.mark.parametrize("dtype", [rd.F32, rd.BF16, rd.F16, rd.I32])
@pytest.mark.parametrize("R,count", [(1, 8), (2, 8), (3, 16), (8, 32), (8, 5)])
def test_reduce_scatter_replay_fold_bruteforce(dtype, R, count):
    w = wi.Workload("t", R, [wi.CollSpec(0, wi.RS, dtype, count)], [[0]] * R, seed=31, cfg=98)
    sends = wi.all_sends(w, 0)
    rep = rd.reduce_scatter_replay(sends, dtype)
    fold = rd.reduce_scatter_fold(sends, dtype)
    for r in range(R):
        assert np.array_equal(rep[r].view(np.uint8), fold[r].view(np.uint8))
        # brute force: scalar loop in the order r+1, r+2, ..., r
        blocks = [s[r * count:(r + 1) * count] for s in sends]
        if dtype == rd.I32:
            want = (np.sum(np.stack([b.astype(np.int64) for b in blocks]), axis=0) + 2**31) % 2**32 - 2**31
            assert np.array_equal(rep[r].astype(np.int64), want)
        elif dtype == rd.F32:
            for i in range(count):
                v = np.float32(blocks[(r + 1) % R][i])
                for j in range(2, R + 1):
                    v = np.float32(v + blocks[(r + j) % R][i])
                assert rep[r][i] == v


@pytest.mark.parametrize("dtype", [rd.F32, rd.BF16])
def test_reduce_scatter_equals_allreduce_chunk_and_gather_identity(dtype):
    R, count = 8, 64           # count*E multiple of 16 so ring chunk == block
    w = wi.Workload("t", R, [wi.CollSpec(0, wi.RS, dtype, count)], [[0]] * R, seed=32, cfg=97)
    sends = wi.all_sends(w, 0)
    rs = rd.reduce_scatter_replay(sends, dtype)
    ar = rd.all_reduce_replay(sends, dtype)[0]
    for r in range(R):
        assert np.array_equal(rs[r], ar[r * count:(r + 1) * count])
    ag = rd.all_gather_replay(rs, dtype)
    assert np.array_equal(ag[3], ar)


def test_dispatch_helpers_agree():
    R = 4
    for kind, dtype, count in [(0, rd.F32, 50), (1, rd.F16, 12), (2, rd.I32, 9), (3, rd.F32, 33)]:
        w = wi.Workload("t", R, [wi.CollSpec(0, kind, dtype, count, root=2)], [[0]] * R, seed=41, cfg=96)
        sends = wi.all_sends(w, 0)
        a = rd.run_replay(kind, sends, dtype, root=2)
        b = rd.run_closed_form(kind, sends, dtype, root=2)
        for r in range(R):
            assert np.array_equal(a[r].view(np.uint8), b[r].view(np.uint8))


@pytest.mark.parametrize("threads", [1, 3, 8])
def test_threaded_replay_gives_the_same_bits(threads):
    """The replay driven by worker threads (the bench's CPU baseline leg) against the round-robin replay and
    the closed form, on ragged sizes and every dtype."""
    for dtype, n in ((rd.F32, 100003), (rd.BF16, 4099), (rd.F16, 70001), (rd.I32, 17)):
        w = wi.Workload("thr", 8, [wi.CollSpec(0, wi.AR, dtype, n)], [[0]] * 8, seed=threads, cfg=71)
        sends = wi.all_sends(w, 0)
        a = rd.all_reduce_replay(sends, dtype)
        b = rd.all_reduce_replay(sends, dtype, threads=threads)
        f = rd.all_reduce_fold(sends, dtype)
        for r in range(8):
            assert np.array_equal(a[r].view(np.uint8), b[r].view(np.uint8))
            assert np.array_equal(b[r].view(np.uint8), f.view(np.uint8))
