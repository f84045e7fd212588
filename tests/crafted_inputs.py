"""Constructed send buffers for the value edge cases of the reducing collectives.

Inputs only (no arithmetic of the method): for every dtype and reducing function, R buffers of n
elements in storage dtype whose folds pass through the places where a reduction kernel can go wrong
without random data ever showing it:

  * gradual underflow: subnormal inputs, subnormal results, results at the normal / subnormal border
    (no flush to zero anywhere on the path);
  * exact cancellation: x and -x on two ranks and signed zeros on the others, so partial results are
    +0 or -0 and the sign rules of IEEE addition decide the bits;
  * values within one binade of the largest finite value whose partial results stay finite in every
    rotation of the fold;
  * constructed round-to-nearest-even ties: 2^p + 1 + 1 ... for a p-bit significand (2^24 for fp32,
    2^8 for bf16, 2^11 for fp16), with the large value also at 2^p + 2 so that a tie rounds up as
    well as down; for the product, (1 + 2^-a)(1 + 2^-b) with a + b = p;
  * equal values and +0 / -0 on several ranks for maximum / minimum;
  * int32 sums and products that wrap.

The five kinds of element are interleaved with period 5 R, and the rank that holds the special
value of element j is j mod R: every ring chunk (a contiguous R-th of the buffer) therefore sees
every kind in every rotation of the fold's starting rank.
"""
from __future__ import annotations

from typing import List

import numpy as np

F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, PROD, MAX, MIN = 0, 1, 2, 3

# significand bits (hidden one included), smallest normal exponent, largest finite exponent
FMT = {F32: (24, -126, 127), BF16: (8, -126, 127), F16: (11, -14, 15)}


def _store(dtype: int, v: np.ndarray) -> np.ndarray:
    """float64 values that are exactly representable in `dtype` -> storage array (bf16: uint16 bits)."""
    if dtype == F32:
        out = v.astype(np.float32)
        assert np.array_equal(out.astype(np.float64), v), "value not representable in fp32"
        return out
    if dtype == F16:
        out = v.astype(np.float16)
        assert np.array_equal(out.astype(np.float64), v), "value not representable in fp16"
        return out
    f = v.astype(np.float32)
    assert np.array_equal(f.astype(np.float64), v)
    bits = f.view(np.uint32)
    assert not np.any(bits & np.uint32(0xffff)), "value not representable in bf16"
    return (bits >> np.uint32(16)).astype(np.uint16)


def _limits(dtype: int):
    p, emin, emax = FMT[dtype]
    d = 2.0 ** (emin - (p - 1))                      # smallest subnormal
    big = (2.0 - 2.0 ** (1 - p)) * 2.0 ** emax       # largest finite
    ulp_big = 2.0 ** (emax - (p - 1))
    return p, emin, emax, d, big, ulp_big


def _float_sum(dtype: int, R: int, n: int, g: np.random.Generator) -> np.ndarray:
    p, emin, emax, d, big, ulp_big = _limits(dtype)
    j = np.arange(n)
    who = j % R                                      # the rank that holds the special value
    typ = (j // R) % 5
    v = np.zeros((R, n), np.float64)
    sign = np.where(g.integers(0, 2, size=n) == 1, -1.0, 1.0)
    rows = np.arange(R)[:, None]
    # 0: ties.  One rank holds +-2^p or +-(2^p + 2), the others hold +-1 (same sign)
    T = 2.0 ** p + 2.0 * g.integers(0, 2, size=n)
    a0 = np.where(rows == who[None, :], (sign * T)[None, :], sign[None, :] * np.ones((R, 1)))
    # 1: subnormals and the border to the normal numbers
    k = g.integers(-7, 8, size=(R, n)).astype(np.float64)
    near = np.where(g.integers(0, 3, size=n) == 0, 1.0, 0.0)       # a third of them start at the smallest normal
    a1 = k * d + np.where(rows == who[None, :], (near * sign * 2.0 ** emin)[None, :], 0.0)
    # 2: exact cancellation: x on one rank, -x on the next but one, signed zeros elsewhere
    mant = 1.0 + g.integers(0, 2 ** (p - 1), size=n) * 2.0 ** (1 - p)
    x = sign * mant * 2.0 ** g.integers(-6, 7, size=n)
    other = (who + 1 + g.integers(0, R - 1, size=n)) % R if R > 1 else who
    zeros = np.where(g.integers(0, 2, size=(R, n)) == 1, -0.0, 0.0)
    a2 = np.where(rows == who[None, :], x[None, :], np.where(rows == other[None, :], -x[None, :], zeros))
    # (a sum is -0 only when every term is: a quarter of these elements hold -0 on every rank, another
    # quarter -0 on every rank but one, which holds +0)
    sel = g.integers(0, 4, size=n)
    a2 = np.where((sel == 0)[None, :], -0.0, a2)
    a2 = np.where((sel == 1)[None, :], np.where(rows == who[None, :], 0.0, -0.0), a2)
    if R == 1:
        a2 = x[None, :].copy()
    # 3: within one binade of the largest finite value; every partial sum stays finite: one rank holds
    # +-(big - k ulp), another -+big/2, the rest at most 2^-12 of it and of the sign opposite to the large one
    top = sign * (big - g.integers(0, 64, size=n) * ulp_big)
    half = -sign * 2.0 ** emax * (2.0 - 2.0 ** (1 - p)) / 2.0
    small = -sign[None, :] * g.integers(0, 4, size=(R, n)) * 2.0 ** (emax - 12)
    a3 = np.where(rows == who[None, :], top[None, :], np.where(rows == other[None, :], half[None, :], small))
    if R == 1:
        a3 = top[None, :].copy()
    # 4: a pool of special values, magnitude at most big / 16
    pool = np.array([0.0, -0.0, d, -d, 2.0 ** emin, -(2.0 ** emin), 2.0 ** emin - d, 1.0, -1.0, 1.0 + 2.0 ** (1 - p),
                     2.0 ** p, 2.0 ** p + 2.0, -(2.0 ** p) - 2.0, 3.0, 2.0 ** (emax - 4), -(2.0 ** (emax - 4)), 0.5, 2.0 ** (emin + p)])
    a4 = pool[g.integers(0, len(pool), size=(R, n))]
    for t, a in enumerate((a0, a1, a2, a3, a4)):
        v[:, typ == t] = a[:, typ == t]
    return v


def _float_prod(dtype: int, R: int, n: int, g: np.random.Generator) -> np.ndarray:
    p, emin, emax, d, big, ulp_big = _limits(dtype)
    j = np.arange(n)
    who = j % R
    typ = (j // R) % 5
    rows = np.arange(R)[:, None]
    other = (who + 1 + g.integers(0, max(R - 1, 1), size=n)) % R
    sign = np.where(g.integers(0, 2, size=(R, n)) == 1, -1.0, 1.0)
    # 0: ties: (1 + 2^-a)(1 + 2^-b) with a + b = p on two ranks, +-1 on the others
    a_ = g.integers(2, p - 2, size=n)
    va, vb = 1.0 + 2.0 ** (-a_.astype(np.float64)), 1.0 + 2.0 ** (-(p - a_).astype(np.float64))
    a0 = np.where(rows == who[None, :], va[None, :], np.where(rows == other[None, :], vb[None, :], 1.0)) * sign
    # 1: products that end subnormal or at the border: exponents that add up to emin - p + 1 .. emin + 1
    tot = g.integers(emin - p + 1, emin + 2, size=n)
    base = np.floor_divide(tot, R)
    rem = tot - base * R
    e = base[None, :] + (rows < rem[None, :])
    m = np.array([1.0, 1.5, 1.25, 1.75])[g.integers(0, 4, size=(R, n))]
    a1 = sign * m * 2.0 ** e.astype(np.float64)
    # (every other one of them: a subnormal input on one rank times small powers of two on the others)
    sub = g.integers(1, 2 ** min(p - 1, 7), size=n) * d
    pw = 2.0 ** g.integers(0, 3, size=(R, n)).astype(np.float64)
    a1b = np.where(rows == who[None, :], sub[None, :], pw) * sign
    a1 = np.where(((j // (5 * R)) % 2 == 0)[None, :], a1, a1b)
    # 2: signed zeros
    z = np.where(g.integers(0, 2, size=n) == 1, -0.0, 0.0)
    vals = np.array([1.0, 2.0, 0.5, 1.5])[g.integers(0, 4, size=(R, n))] * sign
    a2 = np.where(rows == who[None, :], z[None, :], vals)
    # 3: one rank within a binade of the largest finite value, one other +-1 or +-1/2, the rest +-1
    top = big - g.integers(0, 64, size=n) * ulp_big
    halfone = np.array([1.0, 0.5])[g.integers(0, 2, size=n)]
    a3 = np.where(rows == who[None, :], top[None, :], np.where(rows == other[None, :], halfone[None, :], 1.0)) * sign
    # 4: a pool with exponents in -1 .. 1, so that R <= 16 factors stay finite in every dtype
    pool = np.array([1.0, -1.0, 0.5, 2.0, 1.5, 0.75, 1.0 + 2.0 ** (1 - p), 2.0 - 2.0 ** (1 - p), 1.0 - 2.0 ** (-p), 1.25, -1.75])
    a4 = pool[g.integers(0, len(pool), size=(R, n))]
    v = np.zeros((R, n), np.float64)
    for t, a in enumerate((a0, a1, a2, a3, a4)):
        v[:, typ == t] = a[:, typ == t]
    return v


def _float_select(dtype: int, R: int, n: int, g: np.random.Generator) -> np.ndarray:
    p, emin, emax, d, big, ulp_big = _limits(dtype)
    pool = np.array([0.0, -0.0, d, -d, 2.0 ** emin, -(2.0 ** emin), 2.0 ** emin - d, -(2.0 ** emin - d), 1.0, -1.0,
                     1.0 + 2.0 ** (1 - p), big, -big, big - ulp_big, -(big - ulp_big), 2.0 ** p + 2.0])
    v = pool[g.integers(0, len(pool), size=(R, n))]
    j = np.arange(n)
    if R > 1:
        # forced ties: on every other element a second rank repeats the first one's value, or its zero
        # with the other sign
        who, other = j % R, (j % R + 1 + g.integers(0, R - 1, size=n)) % R
        tie = (j // R) % 2 == 0
        src = v[who, j]
        flip = np.where((src == 0.0) & (g.integers(0, 2, size=n) == 1), -1.0, 1.0)
        v[other[tie], j[tie]] = (np.copysign(1.0, src) * flip * np.abs(src))[tie]
    return v


def _int32(op: int, R: int, n: int, g: np.random.Generator) -> np.ndarray:
    lo, hi = -(1 << 31), (1 << 31) - 1
    pool = np.array([hi, lo, hi - 1, lo + 1, -1, 0, 1, 65536, -65536, 3, 46341, 0x7fff0000, -0x12345678], np.int64)
    v = pool[g.integers(0, len(pool), size=(R, n))]
    rnd = g.integers(lo, hi + 1, size=(R, n), dtype=np.int64)
    pick = g.integers(0, 2, size=(R, n)) == 1
    v = np.where(pick, v, rnd)
    if op in (MAX, MIN) and R > 1:
        j = np.arange(n)
        who, other = j % R, (j % R + 1 + g.integers(0, R - 1, size=n)) % R
        tie = (j // R) % 2 == 0
        v[other[tie], j[tie]] = v[who[tie], j[tie]]
    return v.astype(np.int32)


def crafted_sends(dtype: int, op: int, R: int, n: int, seed: int = 0) -> List[np.ndarray]:
    """R send buffers of n elements each (storage dtype) for reducing function `op`."""
    g = np.random.default_rng(np.random.SeedSequence([seed, 7700, dtype, op, R, n]))
    if n == 0:
        return [np.zeros(0, {F32: np.float32, BF16: np.uint16, F16: np.float16, I32: np.int32}[dtype]) for _ in range(R)]
    if dtype == I32:
        v = _int32(op, R, n, g)
        return [np.ascontiguousarray(v[r]) for r in range(R)]
    if op == SUM:
        v = _float_sum(dtype, R, n, g)
    elif op == PROD:
        v = _float_prod(dtype, R, n, g)
    else:
        v = _float_select(dtype, R, n, g)
    return [_store(dtype, np.ascontiguousarray(v[r])) for r in range(R)]
