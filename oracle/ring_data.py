"""CPU oracle, part D: the VALUES a ring collective produces.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file;
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg use it.
It shares no code with the HIP path.

What is modelled (paper Sec. 4.1: a collective is a per-rank sequence of
primitives, each a fusion of send / recv / reduce / copy on the send buffer,
the recv buffer and the send/recv connectors; the input is cut into regular
chunks; Sec. 6: sequences come from the Ring algorithm, Simple protocol).
The paper gives no step table, so the textbook ring is used:

  * rank r sends to (r+1) mod R and receives from (r-1) mod R;
  * ring chunk c of an N-element message is elements
    [min(c*ce, N), min((c+1)*ce, N)) with ce = ceil(N/R) rounded up to a
    multiple of 16 bytes' worth of elements;
  * reduce-scatter phase, step s on rank r: s=0 sends own chunk (r-1);
    0<s<R-1 receives the partial of chunk (r-1-s), adds its own send-buffer
    chunk, forwards; s=R-1 receives the partial of chunk r, adds, keeps;
  * all-gather phase: rank r at step j forwards chunk (r-j);
  * all-reduce fuses the two at the boundary step (recv-reduce-copy-send).

Hence chunk c is the left fold  ((x[c+1] + x[c+2]) + ...) + x[c]  (indices
mod R), one rounding per + in the storage dtype.  FIFO slices and channels of
the GPU path only subdivide a chunk; they never move an element to another
chunk, so the values do not depend on them.

The `reduce` collective (Sec. 4.1 lists it with the others) is the same
reduce phase run along a chain that ends at the root: rank root+1 sends its
whole buffer, the ranks after it receive, combine with their own and forward,
the root receives, combines and keeps.  The root's result is therefore the
left fold  ((x[root+1] (+) x[root+2]) (+) ...) (+) x[root]; the other ranks'
recv buffers are not written.

The reducing function (Sec. 4.1: "a specified reducing function") may be sum,
product, maximum or minimum; `partial (op) own` is evaluated at every hop with
the partial that arrived from the left as the first operand.

Arithmetic (the paper is silent; this is the reading taken): fp32 = one
IEEE binary32 round-to-nearest-even add per hop, gradual underflow; fp16 and
bf16 = widen both operands to fp32, add, round to nearest even back to 16 bits
at every hop (partials travel in the storage dtype); int32 = wraparound.
Product follows the same rule with * for +.  Maximum / minimum select one of
the two operands unchanged:  max = partial if partial > own else own,
min = partial if partial < own else own  (so equal values, +0 / -0 included,
yield the own operand; NaN is outside what is tested).

Two implementations live here on purpose: `*_replay` literally runs R rank
objects exchanging chunks through per-edge queues with the seven primitives;
`*_fold` / `*_definition` write the closed form.  Tests require them to agree
bit for bit, and pin both against brute force, fp64 sums, torch CPU 16-bit
adds and integer-valued inputs.

bf16 buffers are numpy uint16 bit patterns; fp16 = numpy float16; fp32 =
float32; int32 = int32.  dtype codes: 0 fp32, 1 bf16, 2 fp16, 3 int32.
op codes: 0 sum, 1 product, 2 maximum, 3 minimum.  kind codes: 0 all-reduce,
1 all-gather, 2 reduce-scatter, 3 broadcast, 4 reduce.
"""
from __future__ import annotations

from collections import deque
from typing import List, Sequence, Tuple

import numpy as np

F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, PROD, MAX, MIN = 0, 1, 2, 3
ELEM_BYTES = {F32: 4, BF16: 2, F16: 2, I32: 4}


# ----------------------------------------------------------------------------
# storage-dtype arithmetic
# ----------------------------------------------------------------------------
def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 is the upper half of a binary32: widening is exact."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16_bits_rne(x: np.ndarray) -> np.ndarray:
    """Round a binary32 to the nearest bf16, ties to even (finite inputs; NaN kept NaN)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    nan = (u & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    rounded = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x0040), rounded)
    return rounded.astype(np.uint16)


def add_hop(a: np.ndarray, b: np.ndarray, dtype: int) -> np.ndarray:
    """One reduction hop a (+) b with a single rounding in the storage dtype."""
    if dtype == F32:
        return (a.astype(np.float32, copy=False) + b.astype(np.float32, copy=False)).astype(np.float32)
    if dtype == F16:
        return (a.astype(np.float32) + b.astype(np.float32)).astype(np.float16)
    if dtype == BF16:
        return f32_to_bf16_bits_rne(bf16_bits_to_f32(a) + bf16_bits_to_f32(b))
    if dtype == I32:
        return (a.view(np.uint32) + b.view(np.uint32)).view(np.int32)
    raise ValueError(f"dtype {dtype}")


def mul_hop(a: np.ndarray, b: np.ndarray, dtype: int) -> np.ndarray:
    """One product hop a (*) b with a single rounding in the storage dtype."""
    if dtype == F32:
        return (a.astype(np.float32, copy=False) * b.astype(np.float32, copy=False)).astype(np.float32)
    if dtype == F16:
        return (a.astype(np.float32) * b.astype(np.float32)).astype(np.float16)
    if dtype == BF16:
        return f32_to_bf16_bits_rne(bf16_bits_to_f32(a) * bf16_bits_to_f32(b))
    if dtype == I32:
        return (a.view(np.uint32) * b.view(np.uint32)).view(np.int32)
    raise ValueError(f"dtype {dtype}")


def _ordered(a: np.ndarray, dtype: int) -> np.ndarray:
    """The values comparisons are made on (bf16 bit patterns are widened; the rest compare as stored)."""
    return bf16_bits_to_f32(a) if dtype == BF16 else a


def select_hop(a: np.ndarray, b: np.ndarray, dtype: int, want_max: bool) -> np.ndarray:
    """Maximum / minimum hop: the partial `a` if it is strictly greater (smaller) than the own
    value `b`, else `b`; the chosen operand is passed on bit for bit."""
    va, vb = _ordered(a, dtype), _ordered(b, dtype)
    take_a = (va > vb) if want_max else (va < vb)
    return np.where(take_a, a, b).astype(a.dtype)


def op_hop(a: np.ndarray, b: np.ndarray, dtype: int, op: int) -> np.ndarray:
    """partial (op) own for one hop."""
    if op == SUM:
        return add_hop(a, b, dtype)
    if op == PROD:
        return mul_hop(a, b, dtype)
    if op == MAX:
        return select_hop(a, b, dtype, True)
    if op == MIN:
        return select_hop(a, b, dtype, False)
    raise ValueError(f"op {op}")


def to_f64(a: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# ----------------------------------------------------------------------------
# chunking
# ----------------------------------------------------------------------------
def chunk_elems(N: int, R: int, elem_bytes: int) -> int:
    per16 = 16 // elem_bytes
    ce = -(-N // R)
    return -(-ce // per16) * per16


def chunk_bounds(N: int, R: int, elem_bytes: int) -> List[Tuple[int, int]]:
    ce = chunk_elems(N, R, elem_bytes)
    return [(min(c * ce, N), min((c + 1) * ce, N)) for c in range(R)]


# ----------------------------------------------------------------------------
# replay machinery: R ranks, one unbounded queue per ring edge
# ----------------------------------------------------------------------------
class _Rank:
    """One rank's four buffers (Sec. 4.1): send buffer, recv buffer, and the
    send / recv connectors (here: queues towards r+1 and from r-1)."""

    def __init__(self, r, R, sendbuf, recvbuf, dtype, q_in, q_out, op=SUM):
        self.r, self.R, self.dtype, self.op = r, R, dtype, op
        self.sendbuf, self.recvbuf = sendbuf, recvbuf
        self.q_in, self.q_out = q_in, q_out
        self.pc = 0            # index of the next primitive in this rank's sequence
        self.prog = []         # list of (primitive name, src range in sendbuf, dst range in recvbuf)

    # -- the primitives; each returns False if its recv side has nothing to read yet
    def _readable(self):
        return len(self.q_in) > 0

    def send(self, s, d):
        self.q_out.append(self.sendbuf[s[0]:s[1]].copy())
        return True

    def copy_send(self, s, d):
        x = self.sendbuf[s[0]:s[1]].copy()
        self.recvbuf[d[0]:d[1]] = x
        self.q_out.append(x)
        return True

    def copy(self, s, d):
        self.recvbuf[d[0]:d[1]] = self.sendbuf[s[0]:s[1]]
        return True

    def recv_reduce_send(self, s, d):
        if not self._readable():
            return False
        self.q_out.append(op_hop(self.q_in.popleft(), self.sendbuf[s[0]:s[1]], self.dtype, self.op))
        return True

    def recv_reduce_copy_send(self, s, d):
        if not self._readable():
            return False
        x = op_hop(self.q_in.popleft(), self.sendbuf[s[0]:s[1]], self.dtype, self.op)
        self.recvbuf[d[0]:d[1]] = x
        self.q_out.append(x)
        return True

    def recv_reduce_copy(self, s, d):
        if not self._readable():
            return False
        self.recvbuf[d[0]:d[1]] = op_hop(self.q_in.popleft(), self.sendbuf[s[0]:s[1]], self.dtype, self.op)
        return True

    def recv_copy_send(self, s, d):
        if not self._readable():
            return False
        x = self.q_in.popleft()
        self.recvbuf[d[0]:d[1]] = x
        self.q_out.append(x)
        return True

    def recv_copy(self, s, d):
        if not self._readable():
            return False
        self.recvbuf[d[0]:d[1]] = self.q_in.popleft()
        return True

    def step(self) -> bool:
        """Try the next primitive; True if it ran."""
        if self.pc >= len(self.prog):
            return False
        name, s, d = self.prog[self.pc]
        if getattr(self, name)(s, d):
            self.pc += 1
            return True
        return False


def _run(ranks: Sequence[_Rank]) -> None:
    """Round-robin over the ranks until every sequence has finished."""
    while any(k.pc < len(k.prog) for k in ranks):
        moved = False
        for k in ranks:
            while k.step():
                moved = True
        if not moved:
            raise RuntimeError("ring replay stalled: sequences are inconsistent")
    for k in ranks:
        assert len(k.q_in) == 0, "a connector still holds data: something was sent but never received"


def _run_threaded(ranks: Sequence[_Rank], nthreads: int, timeout_s: float = 600.0) -> None:
    """The same sequences with the ranks dealt to `nthreads` worker threads (rank r belongs to thread
    r mod nthreads; one thread per rank when there are enough).  Each thread steps its own ranks and
    yields when none of them can move; only the schedule differs from _run, every rank still runs its
    primitives in order and an edge's queue has one producer and one consumer, so the values are the same.
    For timing the replay on several host cores (numpy releases the interpreter lock inside large array
    operations)."""
    import threading
    import time as _time
    errors: list = []
    deadline = _time.monotonic() + timeout_s

    def work(t):
        mine = [k for k in ranks if k.r % nthreads == t]
        try:
            while any(k.pc < len(k.prog) for k in mine):
                moved = False
                for k in mine:
                    while k.step():
                        moved = True
                if not moved:
                    if errors or _time.monotonic() > deadline:
                        raise RuntimeError("threaded ring replay stalled")
                    _time.sleep(0)
        except Exception as e:   # noqa: BLE001
            errors.append(e)

    ts = [threading.Thread(target=work, args=(t,)) for t in range(nthreads)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    if errors:
        raise errors[0]
    for k in ranks:
        assert len(k.q_in) == 0, "a connector still holds data: something was sent but never received"


def _make_ranks(sends, recv_elems, dtype, op=SUM):
    R = len(sends)
    queues = [deque() for _ in range(R)]          # queues[r] = edge r -> r+1
    recvs = [np.zeros(recv_elems, dtype=sends[0].dtype) for _ in range(R)]
    ranks = [_Rank(r, R, sends[r], recvs[r], dtype, queues[(r - 1) % R], queues[r], op) for r in range(R)]
    return ranks, recvs


# ----------------------------------------------------------------------------
# all-reduce
# ----------------------------------------------------------------------------
def all_reduce_replay(sends: Sequence[np.ndarray], dtype: int, op: int = SUM, threads: int = 0) -> List[np.ndarray]:
    """threads = 0: the ranks are stepped round-robin by the caller's thread; threads > 0: by that many
    worker threads (same values, see _run_threaded)."""
    R, N = len(sends), len(sends[0])
    ranks, recvs = _make_ranks(sends, N, dtype, op)
    if R == 1:
        ranks[0].prog = [("copy", (0, N), (0, N))]
        _run(ranks)
        return recvs
    cb = chunk_bounds(N, R, ELEM_BYTES[dtype])
    for k in ranks:
        r = k.r
        ch = lambda j: cb[j % R]
        k.prog.append(("send", ch(r - 1), None))
        for s in range(1, R - 1):
            k.prog.append(("recv_reduce_send", ch(r - 1 - s), None))
        k.prog.append(("recv_reduce_copy_send", ch(r), ch(r)))
        for j in range(1, R - 1):
            k.prog.append(("recv_copy_send", None, ch(r - j)))
        k.prog.append(("recv_copy", None, ch(r + 1)))
        # primitives without a send-buffer / recv-buffer side get a dummy range
        k.prog = [(n, s or (0, 0), d or (0, 0)) for n, s, d in k.prog]
    if threads > 0:
        _run_threaded(ranks, min(threads, R))
    else:
        _run(ranks)
    return recvs


def fold_rotated(blocks: Sequence[np.ndarray], start: int, dtype: int, op: int = SUM) -> np.ndarray:
    """((b[start] (op) b[start+1]) (op) ...) (op) b[start-1], indices mod R."""
    R = len(blocks)
    v = blocks[start % R].copy()
    for j in range(1, R):
        v = op_hop(v, blocks[(start + j) % R], dtype, op)
    return v


def all_reduce_fold(sends: Sequence[np.ndarray], dtype: int, op: int = SUM) -> np.ndarray:
    """Closed form: the buffer every rank ends with."""
    R, N = len(sends), len(sends[0])
    out = np.zeros(N, dtype=sends[0].dtype)
    if R == 1:
        out[:] = sends[0]
        return out
    for c, (lo, hi) in enumerate(chunk_bounds(N, R, ELEM_BYTES[dtype])):
        if hi > lo:
            out[lo:hi] = fold_rotated([x[lo:hi] for x in sends], c + 1, dtype, op)
    return out


# ----------------------------------------------------------------------------
# reduce-scatter: send holds R blocks of `count`; rank r ends with block r reduced
# ----------------------------------------------------------------------------
def reduce_scatter_replay(sends: Sequence[np.ndarray], dtype: int, op: int = SUM) -> List[np.ndarray]:
    R = len(sends)
    count = len(sends[0]) // R
    ranks, recvs = _make_ranks(sends, count, dtype, op)
    blk = lambda j: ((j % R) * count, (j % R + 1) * count)
    for k in ranks:
        r = k.r
        if R == 1:
            k.prog = [("copy", blk(0), (0, count))]
            continue
        k.prog.append(("send", blk(r - 1), (0, 0)))
        for s in range(1, R - 1):
            k.prog.append(("recv_reduce_send", blk(r - 1 - s), (0, 0)))
        k.prog.append(("recv_reduce_copy", blk(r), (0, count)))
    _run(ranks)
    return recvs


def reduce_scatter_fold(sends: Sequence[np.ndarray], dtype: int, op: int = SUM) -> List[np.ndarray]:
    R = len(sends)
    count = len(sends[0]) // R
    return [fold_rotated([x[r * count:(r + 1) * count] for x in sends], r + 1, dtype, op) for r in range(R)]


# ----------------------------------------------------------------------------
# all-gather: every rank ends with the concatenation of all send buffers
# ----------------------------------------------------------------------------
def all_gather_replay(sends: Sequence[np.ndarray], dtype: int) -> List[np.ndarray]:
    R, count = len(sends), len(sends[0])
    ranks, recvs = _make_ranks(sends, R * count, dtype)
    blk = lambda j: ((j % R) * count, (j % R + 1) * count)
    for k in ranks:
        r = k.r
        if R == 1:
            k.prog = [("copy", (0, count), blk(0))]
            continue
        k.prog.append(("copy_send", (0, count), blk(r)))
        for j in range(1, R - 1):
            k.prog.append(("recv_copy_send", (0, 0), blk(r - j)))
        k.prog.append(("recv_copy", (0, 0), blk(r + 1)))
    _run(ranks)
    return recvs


def all_gather_definition(sends: Sequence[np.ndarray]) -> np.ndarray:
    return np.concatenate(list(sends))


# ----------------------------------------------------------------------------
# broadcast: chain root -> root+1 -> ... -> root-1; root also fills its own recv buffer
# ----------------------------------------------------------------------------
def broadcast_replay(sends: Sequence[np.ndarray], root: int, dtype: int) -> List[np.ndarray]:
    R, N = len(sends), len(sends[0])
    ranks, recvs = _make_ranks(sends, N, dtype)
    for k in ranks:
        pos = (k.r - root) % R          # distance from the root along the ring
        if R == 1:
            k.prog = [("copy", (0, N), (0, N))]
        elif pos == 0:
            k.prog = [("copy_send", (0, N), (0, N))]
        elif pos == R - 1:
            k.prog = [("recv_copy", (0, 0), (0, N))]
        else:
            k.prog = [("recv_copy_send", (0, 0), (0, N))]
    _run(ranks)
    return recvs


def broadcast_definition(sends: Sequence[np.ndarray], root: int) -> np.ndarray:
    return sends[root].copy()


# ----------------------------------------------------------------------------
# reduce: chain root+1 -> root+2 -> ... -> root; only the root's recv buffer is written
# ----------------------------------------------------------------------------
def reduce_replay(sends: Sequence[np.ndarray], root: int, dtype: int, op: int = SUM) -> List[np.ndarray]:
    R, N = len(sends), len(sends[0])
    ranks, recvs = _make_ranks(sends, N, dtype, op)
    for k in ranks:
        pos = (k.r - root - 1) % R      # place in the chain: 0 = first sender, R-1 = the root
        if R == 1:
            k.prog = [("copy", (0, N), (0, N))]
        elif pos == 0:
            k.prog = [("send", (0, N), (0, 0))]
        elif pos == R - 1:
            k.prog = [("recv_reduce_copy", (0, N), (0, N))]
        else:
            k.prog = [("recv_reduce_send", (0, N), (0, 0))]
    _run(ranks)
    return recvs


def reduce_fold(sends: Sequence[np.ndarray], root: int, dtype: int, op: int = SUM) -> np.ndarray:
    """Closed form: what the root ends with."""
    return fold_rotated(list(sends), root + 1, dtype, op)


# ----------------------------------------------------------------------------
# order-independent references and dispatch
# ----------------------------------------------------------------------------
def sum_f64(blocks: Sequence[np.ndarray], dtype: int) -> np.ndarray:
    acc = np.zeros(len(blocks[0]), dtype=np.float64)
    for b in blocks:
        acc += to_f64(b, dtype)
    return acc


def abs_sum_f64(blocks: Sequence[np.ndarray], dtype: int) -> np.ndarray:
    acc = np.zeros(len(blocks[0]), dtype=np.float64)
    for b in blocks:
        acc += np.abs(to_f64(b, dtype))
    return acc


def run_replay(kind: int, sends: Sequence[np.ndarray], dtype: int, root: int = 0, op: int = SUM) -> List[np.ndarray]:
    """kind: 0 all-reduce, 1 all-gather, 2 reduce-scatter, 3 broadcast, 4 reduce.  Returns every rank's
    recv buffer (reduce: zeros on the ranks that are not the root, which the collective does not write)."""
    if kind == 0:
        return all_reduce_replay(sends, dtype, op)
    if kind == 1:
        return all_gather_replay(sends, dtype)
    if kind == 2:
        return reduce_scatter_replay(sends, dtype, op)
    if kind == 3:
        return broadcast_replay(sends, root, dtype)
    if kind == 4:
        return reduce_replay(sends, root, dtype, op)
    raise ValueError(f"kind {kind}")


def run_closed_form(kind: int, sends: Sequence[np.ndarray], dtype: int, root: int = 0, op: int = SUM) -> List[np.ndarray]:
    R = len(sends)
    if kind == 0:
        v = all_reduce_fold(sends, dtype, op)
        return [v] * R
    if kind == 1:
        v = all_gather_definition(sends)
        return [v] * R
    if kind == 2:
        return reduce_scatter_fold(sends, dtype, op)
    if kind == 3:
        v = broadcast_definition(sends, root)
        return [v] * R
    if kind == 4:
        v = reduce_fold(sends, root, dtype, op)
        zero = np.zeros_like(v)
        return [v if r == root % R else zero for r in range(R)]
    raise ValueError(f"kind {kind}")
