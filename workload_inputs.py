"""Seeded synthetic inputs for the collective workloads.

This module is the only code shared by the CPU oracle's tests and the GPU
path's tests/bench.  It holds no arithmetic of the method itself: it only
draws random buffers, sizes, kinds, issue orders and submission delays, with
the shapes of the five benchmark configurations (circular wait, size sweep,
gradient buckets in random order, mixed collectives, many small all-reduces).

Encodings (shared with the C ABI enums, restated here as plain integers):
  kind : 0 all-reduce, 1 all-gather, 2 reduce-scatter, 3 broadcast, 4 reduce
  op   : 0 sum, 1 product, 2 maximum, 3 minimum
  dtype: 0 fp32, 1 bf16 (carried as uint16 bit patterns), 2 fp16, 3 int32

Count convention: all-reduce / broadcast / reduce: elements per rank; all-gather:
elements each rank contributes (recv holds R*count); reduce-scatter: elements
each rank receives (send holds R*count).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

AR, AG, RS, BC, RD = 0, 1, 2, 3, 4
SUM, PROD, MAX, MIN = 0, 1, 2, 3
F32, BF16, F16, I32 = 0, 1, 2, 3

KIND_NAMES = {AR: "all_reduce", AG: "all_gather", RS: "reduce_scatter", BC: "broadcast", RD: "reduce"}
OP_NAMES = {SUM: "sum", PROD: "prod", MAX: "max", MIN: "min"}
DTYPE_NAMES = {F32: "fp32", BF16: "bf16", F16: "fp16", I32: "int32"}
ELEM_BYTES = {F32: 4, BF16: 2, F16: 2, I32: 4}
NP_STORAGE = {F32: np.float32, BF16: np.uint16, F16: np.float16, I32: np.int32}

KiB = 1 << 10
MiB = 1 << 20


@dataclass
class CollSpec:
    coll_id: int
    kind: int
    dtype: int
    count: int
    root: int = 0
    op: int = 0

    def send_elems(self, R: int) -> int:
        return self.count * R if self.kind == RS else self.count

    def recv_elems(self, R: int) -> int:
        return self.count * R if self.kind == AG else self.count


@dataclass
class Workload:
    name: str
    R: int
    colls: List[CollSpec]
    # orders[r] = the sequence of coll indices (into colls) rank r submits
    orders: List[List[int]]
    # delays_us[r][j] = host delay before rank r's j-th submission
    delays_us: List[List[float]] = field(default_factory=list)
    value_kind: str = "normal"      # "normal" | "small_int"
    sigma: float = 1.0
    seed: int = 0
    cfg: int = 0


def _rng(seed: int, cfg: int, coll: int, rank: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, cfg, coll, rank]))


def _f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Library conversion (torch CPU, round-to-nearest-even) of fp32 to bf16 bit patterns."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def make_send(w: Workload, ci: int, rank: int) -> np.ndarray:
    """The send buffer of rank `rank` for collective index `ci`, in storage dtype."""
    c = w.colls[ci]
    n = c.send_elems(w.R)
    g = _rng(w.seed, w.cfg, ci, rank)
    if c.dtype == I32:
        return g.integers(-(1 << 20), (1 << 20) + 1, size=n, dtype=np.int64).astype(np.int32)
    if w.value_kind == "small_int":
        v = g.integers(-8, 9, size=n).astype(np.float32)
    else:
        v = (g.standard_normal(size=n, dtype=np.float32) * np.float32(w.sigma)).astype(np.float32)
    if c.dtype == F32:
        return v
    if c.dtype == F16:
        return v.astype(np.float16)
    if c.dtype == BF16:
        return _f32_to_bf16_bits(v)
    raise ValueError(c.dtype)


def all_sends(w: Workload, ci: int) -> List[np.ndarray]:
    return [make_send(w, ci, r) for r in range(w.R)]


def _perm_orders(seed: int, cfg: int, R: int, n: int) -> List[List[int]]:
    return [list(map(int, _rng(seed, cfg, 1 << 20, r).permutation(n))) for r in range(R)]


def _round_down(x: int, m: int) -> int:
    return max(m, (x // m) * m)


# --------------------------------------------------------------------------
# configuration 1: circular wait, R = 2, two all-reduces in opposite orders
# --------------------------------------------------------------------------
def config1(order0=(0, 1), order1=(1, 0), n: int = 1024, seed: int = 0) -> Workload:
    colls = [CollSpec(0, AR, F32, n), CollSpec(1, AR, F32, n)]
    return Workload("cfg1_circular_wait", 2, colls, [list(order0), list(order1)],
                    value_kind="small_int", seed=seed, cfg=1)


# --------------------------------------------------------------------------
# configuration 2: one fp32 all-reduce over 8 ranks, per-rank message bytes given
# --------------------------------------------------------------------------
CONFIG2_SIZES = [1 << p for p in range(13, 29)]   # 8 KiB .. 256 MiB


def config2(msg_bytes: int, seed: int = 0, R: int = 8, dtype: int = F32) -> Workload:
    n = msg_bytes // ELEM_BYTES[dtype]
    colls = [CollSpec(0, AR, dtype, n)]
    return Workload(f"cfg2_allreduce_{msg_bytes}B", R, colls, [[0] for _ in range(R)],
                    seed=seed, cfg=2)


# --------------------------------------------------------------------------
# configuration 3: bf16 gradient buckets, each rank its own random order
# --------------------------------------------------------------------------
def config3(n_buckets: int = 16, bucket_bytes: int = 25 * MiB, seed: int = 0, R: int = 8) -> Workload:
    n = bucket_bytes // 2
    colls = [CollSpec(i, AR, BF16, n) for i in range(n_buckets)]
    return Workload("cfg3_bf16_buckets", R, colls, _perm_orders(seed, 3, R, n_buckets),
                    sigma=1e-2, seed=seed, cfg=3)


# --------------------------------------------------------------------------
# configuration 4: mixed kinds / dtypes / sizes, random orders, staggered submits
# --------------------------------------------------------------------------
def config4(n_colls: int = 64, min_bytes: int = 4 * KiB, max_bytes: int = 64 * MiB,
            seed: int = 0, R: int = 8) -> Workload:
    g = _rng(seed, 4, 1 << 21, 0)
    colls = []
    for i in range(n_colls):
        kind = int(g.integers(0, 4))
        dtype = [F32, F16, I32][int(g.integers(0, 3))]
        size = int(np.exp(g.uniform(np.log(min_bytes), np.log(max_bytes))))
        size = _round_down(size, R * 16)            # bytes of the largest per-rank buffer
        elems = size // ELEM_BYTES[dtype]
        root = int(g.integers(0, R))
        count = elems // R if kind in (AG, RS) else elems
        colls.append(CollSpec(i, kind, dtype, count, root if kind == BC else 0))
    orders = _perm_orders(seed, 4, R, n_colls)
    delays = [list(map(float, _rng(seed, 4, 1 << 22, r).uniform(0.0, 50.0, size=n_colls)))
              for r in range(R)]
    return Workload("cfg4_mixed", R, colls, orders, delays_us=delays, seed=seed, cfg=4)


# --------------------------------------------------------------------------
# configuration 5: many small fp32 all-reduces, random orders, continuous submit
# --------------------------------------------------------------------------
def config5(n_colls: int = 1024, min_bytes: int = 4 * KiB, max_bytes: int = 64 * KiB,
            seed: int = 0, R: int = 8) -> Workload:
    g = _rng(seed, 5, 1 << 21, 0)
    colls = []
    for i in range(n_colls):
        size = int(np.exp(g.uniform(np.log(min_bytes), np.log(max_bytes))))
        size = _round_down(size, R * 16)
        colls.append(CollSpec(i, AR, F32, size // 4))
    return Workload("cfg5_small_allreduces", R, colls, _perm_orders(seed, 5, R, n_colls),
                    seed=seed, cfg=5)
