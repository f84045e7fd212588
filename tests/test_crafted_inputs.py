"""The constructed inputs of the value edge-case GPU test reach what they are built for: checked
here on the CPU, against the oracle, so that the GPU comparison is not vacuous."""
import numpy as np
import pytest

from oracle import ring_data as rd
from tests import crafted_inputs as ci

FLOATS = [rd.F32, rd.BF16, rd.F16]


def _f64(a, dtype):
    return rd.to_f64(a, dtype)


def _is_subnormal(x64, dtype):
    _, emin, _ = ci.FMT[dtype]
    return (x64 != 0) & (np.abs(x64) < 2.0 ** emin)


def _neg_zero(x64):
    return (x64 == 0) & np.signbit(x64)


@pytest.mark.parametrize("R", [3, 8])
@pytest.mark.parametrize("op", [rd.SUM, rd.PROD, rd.MAX, rd.MIN])
@pytest.mark.parametrize("dtype", FLOATS)
def test_float_cases_are_finite_and_hit_their_targets(dtype, op, R):
    n = 5 * R * 300 + 17
    sends = ci.crafted_sends(dtype, op, R, n, seed=1)
    want = rd.all_reduce_fold(sends, dtype, op)
    w64 = _f64(want, dtype)
    assert np.all(np.isfinite(w64))                       # NaN / Inf are outside what is tested
    for s in sends:
        assert np.all(np.isfinite(_f64(s, dtype)))
    ins = np.stack([_f64(s, dtype) for s in sends])
    assert _is_subnormal(ins, dtype).sum() > n // 25       # subnormal inputs
    assert _is_subnormal(w64, dtype).sum() > n // 50       # subnormal results
    assert _neg_zero(ins).sum() > 0
    p, emin, emax = ci.FMT[dtype]
    assert (np.abs(ins) >= 2.0 ** emax).sum() > n // 20    # inputs in the top binade
    if op in (rd.SUM, rd.PROD):
        assert (w64 == 0).sum() > 0 and _neg_zero(w64).sum() > 0 and ((w64 == 0) & ~np.signbit(w64)).sum() > 0
        assert (np.abs(w64) >= 2.0 ** (emax - 1)).sum() > n // 20    # results within a binade or two of the top
    else:
        assert _neg_zero(w64).sum() > 0 and ((w64 == 0) & ~np.signbit(w64)).sum() > 0
        assert (np.abs(w64) == np.abs(ins).max()).sum() > 0


@pytest.mark.parametrize("R", [3, 8])
@pytest.mark.parametrize("dtype", FLOATS)
def test_sum_and_product_cases_contain_exact_ties_in_every_chunk(dtype, R):
    """A hop is a tie when the exact result lies halfway between two neighbouring values of the dtype:
    replay the rotated fold in fp64 next to the oracle's and count them per ring chunk, both directions
    (ties that round the magnitude down and ties that round it up)."""
    n = 5 * R * 200 + 3
    eb = rd.ELEM_BYTES[dtype]
    p, emin, emax = ci.FMT[dtype]
    for op in (rd.SUM, rd.PROD):
        sends = ci.crafted_sends(dtype, op, R, n, seed=2)
        for c, (lo, hi) in enumerate(rd.chunk_bounds(n, R, eb)):
            if hi - lo < 5 * R:
                continue
            order = [(c + 1 + k) % R for k in range(R)]
            part = sends[order[0]][lo:hi]
            down = up = 0
            for r in order[1:]:
                own = sends[r][lo:hi]
                a, b = _f64(part, dtype), _f64(own, dtype)
                exact = a + b if op == rd.SUM else a * b      # exact in fp64: operands have at most 24 bits
                part = rd.op_hop(part, own, dtype, op)
                got = _f64(part, dtype)
                err = np.abs(got - exact)
                mag = np.maximum(np.abs(exact), 2.0 ** emin)
                half_ulp = 2.0 ** (np.floor(np.log2(mag)) - (p - 1)) / 2
                tie = (err > 0) & (err == half_ulp)
                down += int((tie & (np.abs(got) < np.abs(exact))).sum())
                up += int((tie & (np.abs(got) > np.abs(exact))).sum())
            assert down > 0 and up > 0, (dtype, op, c, down, up)


@pytest.mark.parametrize("op", [rd.SUM, rd.PROD, rd.MAX, rd.MIN])
def test_int32_cases_wrap_and_tie(op):
    R, n = 8, 4001
    sends = ci.crafted_sends(rd.I32, op, R, n, seed=3)
    want = rd.all_reduce_fold(sends, rd.I32, op)
    big = [s.astype(object) for s in sends]
    if op == rd.SUM:
        exact = sum(big)
        assert (np.array([abs(int(x)) >= 2 ** 31 for x in exact])).sum() > n // 10       # sums that wrap
    elif op == rd.PROD:
        exact = big[0]
        for b in big[1:]:
            exact = exact * b
        assert (np.array([abs(int(x)) >= 2 ** 31 for x in exact])).sum() > n // 10
    else:
        st = np.stack(sends)
        ext = st.max(axis=0) if op == rd.MAX else st.min(axis=0)
        assert np.array_equal(want, ext)
        assert ((st == ext[None, :]).sum(axis=0) > 1).sum() > n // 10                    # ties between ranks
        return
    wrapped = np.array([((int(x) + 2 ** 31) % 2 ** 32) - 2 ** 31 for x in exact], np.int64).astype(np.int32)
    assert np.array_equal(want, wrapped)
