"""Pins for the oracle's `reduce` collective and its product / maximum / minimum reducing
functions (oracle/ring_data.py); CPU only.

What the oracle is checked against here, none of it the oracle itself: numpy's order-independent
`maximum.reduce` / `minimum.reduce`, exact integer products in Python integers, torch CPU 16-bit
multiplication, fp64 products with the (R-1)-rounding error bound, scalar brute force in the
chain order, and the definition "only the root's recv buffer is written".
"""
import itertools

import numpy as np
import pytest
import torch

import workload_inputs as wi
from oracle import ring_data as rd


def _sends(R, n, dtype, seed=0, value_kind="normal", sigma=1.0):
    w = wi.Workload("t", R, [wi.CollSpec(0, wi.AR, dtype, n)], [[0]] * R, sigma=sigma, seed=seed, cfg=98,
                    value_kind=value_kind)
    return wi.all_sends(w, 0)


def _as_f64(x, dtype):
    return rd.to_f64(x, dtype)


# ---------------------------------------------------------------- one hop
@pytest.mark.parametrize("dtype,tdt", [(rd.BF16, torch.bfloat16), (rd.F16, torch.float16)])
def test_16bit_product_hop_matches_torch_cpu_mul(dtype, tdt):
    a, b = _sends(2, 200000, dtype, seed=3)
    ours = rd.mul_hop(a, b, dtype)
    ta = torch.from_numpy(a.view(np.int16)).view(tdt)
    tb = torch.from_numpy(b.view(np.int16)).view(tdt)
    theirs = (ta * tb).view(torch.int16).numpy()
    assert np.array_equal(ours.view(np.int16), theirs)


def test_fp32_product_hop_is_one_multiplication_correctly_rounded():
    a, b = _sends(2, 100000, rd.F32, seed=4)
    exact = a.astype(np.float64) * b.astype(np.float64)          # exact: 24 x 24 bits fit in 53
    assert np.array_equal(rd.mul_hop(a, b, rd.F32), exact.astype(np.float32))


def test_int32_product_hop_wraps_like_python_integers():
    a, b = _sends(2, 5000, rd.I32, seed=5)
    got = rd.mul_hop(a, b, rd.I32)
    for i in range(0, 5000, 7):
        want = (int(a[i]) * int(b[i]) + 2**31) % 2**32 - 2**31
        assert int(got[i]) == want


@pytest.mark.parametrize("dtype", [rd.F32, rd.BF16, rd.F16, rd.I32])
def test_select_hop_returns_an_operand_and_ties_go_to_own(dtype):
    a, b = _sends(2, 50000, dtype, seed=6)
    b[:1000] = a[:1000]                                           # exact ties
    for want_max in (True, False):
        got = rd.select_hop(a, b, dtype, want_max)
        va, vb, vg = _as_f64(a, dtype), _as_f64(b, dtype), _as_f64(got, dtype)
        ref = np.maximum(va, vb) if want_max else np.minimum(va, vb)
        assert np.array_equal(vg, ref)
        assert np.array_equal(got[:1000], b[:1000])


def test_select_hop_signed_zero_rule():
    # +0 and -0 compare equal: the own operand (second argument) is passed on, bit for bit
    pz, nz = np.array([0.0], np.float32), np.array([-0.0], np.float32)
    for want_max in (True, False):
        assert np.signbit(rd.select_hop(pz, nz, rd.F32, want_max))[0]
        assert not np.signbit(rd.select_hop(nz, pz, rd.F32, want_max))[0]


# ---------------------------------------------------------------- folds with an op
@pytest.mark.parametrize("kindname", ["allreduce", "reduce_scatter", "reduce"])
@pytest.mark.parametrize("dtype", [rd.F32, rd.BF16, rd.F16, rd.I32])
@pytest.mark.parametrize("op", [rd.MAX, rd.MIN])
def test_max_min_equal_the_order_independent_library_reduction(kindname, dtype, op):
    R, n = 5, 1003
    red = np.maximum.reduce if op == rd.MAX else np.minimum.reduce
    if kindname == "allreduce":
        sends = _sends(R, n, dtype, seed=7)
        want = red([_as_f64(x, dtype) for x in sends])
        for out in rd.all_reduce_replay(sends, dtype, op):
            assert np.array_equal(_as_f64(out, dtype), want)
        assert np.array_equal(_as_f64(rd.all_reduce_fold(sends, dtype, op), dtype), want)
    elif kindname == "reduce_scatter":
        sends = _sends(R, n * R, dtype, seed=8)
        want = red([_as_f64(x, dtype) for x in sends])
        outs = rd.reduce_scatter_replay(sends, dtype, op)
        for r in range(R):
            assert np.array_equal(_as_f64(outs[r], dtype), want[r * n:(r + 1) * n])
    else:
        sends = _sends(R, n, dtype, seed=9)
        want = red([_as_f64(x, dtype) for x in sends])
        for root in range(R):
            outs = rd.reduce_replay(sends, root, dtype, op)
            assert np.array_equal(_as_f64(outs[root], dtype), want)


@pytest.mark.parametrize("R", [2, 3, 8])
def test_product_of_small_integers_is_exact(R):
    # factors in {-2,-1,1,2}: every partial product is a power of two times +-1, exact in all dtypes
    g = np.random.default_rng(11)
    n = 777
    ints = [g.choice(np.array([-2, -1, 1, 2]), size=n) for _ in range(R)]
    exact = np.prod(np.stack(ints).astype(np.int64), axis=0)
    for dtype, conv in ((rd.F32, lambda v: v.astype(np.float32)), (rd.F16, lambda v: v.astype(np.float16)),
                        (rd.I32, lambda v: v.astype(np.int32)),
                        (rd.BF16, lambda v: rd.f32_to_bf16_bits_rne(v.astype(np.float32)))):
        sends = [conv(v) for v in ints]
        for out in rd.all_reduce_replay(sends, dtype, rd.PROD):
            assert np.array_equal(_as_f64(out, dtype), exact.astype(np.float64))
        for root in (0, R - 1):
            assert np.array_equal(_as_f64(rd.reduce_replay(sends, root, dtype, rd.PROD)[root], dtype),
                                  exact.astype(np.float64))


@pytest.mark.parametrize("dtype,u", [(rd.F32, 2.0**-24), (rd.F16, 2.0**-11), (rd.BF16, 2.0**-8)])
def test_product_error_bound_vs_fp64(dtype, u):
    R, n = 8, 4000
    sends = _sends(R, n, dtype, seed=12)
    # keep magnitudes near 1 so that nothing overflows or goes subnormal in fp16
    sends = [s if dtype != rd.F16 else (np.sign(s.astype(np.float32)) * (0.5 + np.abs(s.astype(np.float32)) % 1.0)).astype(np.float16)
             for s in sends]
    exact = np.prod(np.stack([_as_f64(x, dtype) for x in sends]), axis=0)
    got = _as_f64(rd.all_reduce_fold(sends, dtype, rd.PROD), dtype)
    bound = ((1 + u) ** (R - 1) - 1) * np.abs(exact) + 1e-300
    assert np.all(np.abs(got - exact) <= bound * 1.0000001)


def test_int32_product_fold_matches_python_integers_with_overflow():
    R, n = 4, 300
    sends = _sends(R, n, rd.I32, seed=13)
    out = rd.all_reduce_fold(sends, rd.I32, rd.PROD)
    for i in range(n):
        v = 1
        for r in range(R):
            v *= int(sends[r][i])
        assert int(out[i]) == (v + 2**31) % 2**32 - 2**31      # wraparound product does not depend on the order


# ---------------------------------------------------------------- the reduce collective
def _brute_reduce_scalar(sends, root, dtype, op):
    """Element by element along the chain root+1, root+2, ..., root; scalar operations only."""
    R, N = len(sends), len(sends[0])
    out = np.zeros(N, dtype=sends[0].dtype)
    order = [(root + 1 + j) % R for j in range(R)]
    for i in range(N):
        if dtype == rd.I32:
            v = int(sends[order[0]][i])
            for r in order[1:]:
                x = int(sends[r][i])
                if op == rd.SUM:
                    v = (v + x + 2**31) % 2**32 - 2**31
                elif op == rd.PROD:
                    v = (v * x + 2**31) % 2**32 - 2**31
                elif op == rd.MAX:
                    v = v if v > x else x
                else:
                    v = v if v < x else x
            out[i] = v
        else:
            cast = np.float32 if dtype == rd.F32 else np.float16
            v = cast(sends[order[0]][i])
            for r in order[1:]:
                x = cast(sends[r][i])
                if op == rd.SUM:
                    v = cast(np.float64(v) + np.float64(x))       # exact in fp64, then one rounding
                elif op == rd.PROD:
                    v = cast(np.float64(v) * np.float64(x))
                elif op == rd.MAX:
                    v = v if v > x else x
                else:
                    v = v if v < x else x
            out[i] = v
    return out


@pytest.mark.parametrize("dtype", [rd.F32, rd.F16, rd.I32])
@pytest.mark.parametrize("op", [rd.SUM, rd.PROD, rd.MAX, rd.MIN])
@pytest.mark.parametrize("R,root", [(2, 0), (3, 2), (5, 1)])
def test_reduce_replay_fold_bruteforce_agree(dtype, op, R, root):
    n = 61
    sends = _sends(R, n, dtype, seed=20 + R)
    outs = rd.reduce_replay(sends, root, dtype, op)
    want = _brute_reduce_scalar(sends, root, dtype, op)
    assert np.array_equal(outs[root].view(np.uint8), want.view(np.uint8))
    assert np.array_equal(rd.reduce_fold(sends, root, dtype, op).view(np.uint8), want.view(np.uint8))


@pytest.mark.parametrize("R", [1, 2, 4, 8])
def test_reduce_writes_only_the_root_and_sums_integers_exactly(R):
    n = 500
    sends = _sends(R, n, rd.F32, seed=30, value_kind="small_int")
    exact = np.sum(np.stack(sends).astype(np.int64), axis=0)
    for root in range(R):
        outs = rd.reduce_replay(sends, root, rd.F32, rd.SUM)
        assert np.array_equal(outs[root].astype(np.int64), exact)
        for r in range(R):
            if r != root:
                assert not outs[r].any()                          # never written


def test_reduce_is_the_root_chunk_rule_of_reduce_scatter():
    # reduce-scatter block r is reduced along the chain that ends at rank r: the same fold as reduce(root = r)
    R, n = 6, 96
    sends = _sends(R, n * R, rd.BF16, seed=31)
    rs = rd.reduce_scatter_replay(sends, rd.BF16)
    for r in range(R):
        blocks = [x[r * n:(r + 1) * n] for x in sends]
        assert np.array_equal(rd.reduce_replay(blocks, r, rd.BF16)[r], rs[r])


def test_planted_operand_order_mistake_is_caught_by_the_tie_rule():
    # swapping partial and own in the selection would pass on the partial at a tie
    a = np.array([0.0, 1.0], np.float32)
    b = np.array([-0.0, 1.0], np.float32)
    wrong = np.where(b > a, b, a)                                 # "own (op) partial"
    right = rd.select_hop(a, b, rd.F32, True)
    assert np.signbit(right[0]) and not np.signbit(wrong[0])


def test_dispatch_covers_reduce_and_ops():
    R, n = 4, 256
    sends = _sends(R, n, rd.F32, seed=40)
    for op in (rd.SUM, rd.PROD, rd.MAX, rd.MIN):
        a = rd.run_replay(4, sends, rd.F32, root=2, op=op)
        b = rd.run_closed_form(4, sends, rd.F32, root=2, op=op)
        for r in range(R):
            assert np.array_equal(a[r], b[r])
        a = rd.run_replay(0, sends, rd.F32, op=op)
        b = rd.run_closed_form(0, sends, rd.F32, op=op)
        for r in range(R):
            assert np.array_equal(a[r], b[r])
