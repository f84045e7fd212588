"""CPU oracle, part S: a tick model of the daemon kernel's scheduler (liveness, not speed).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path may import this file.
It shares no code with the HIP path.

The model follows the paper's scheduling algorithm (Alg. 1, Sec. 4.3) for R ranks,
one daemon ("block") per rank:

    while not exit:
        fetch SQE (FIFO order policy)            -- Sec. 4.3 "FIFO Ordering"
        set initial spin thresholds by position  -- largest at the queue front
        for collective in task queue:
            load its context
            for primitive in collective:
                two-phase blocking execute       -- Sec. 4.2 (3): poll <= threshold times
                success -> raise the threshold of the following primitives
                failure -> preempt, (lazily) save dynamic context, next collective
            complete -> CQE

A collective's per-rank program is the ring primitive sequence (Sec. 4.1) repeated
once per slice ("round"); the dynamic context is (round, primitive index), the pair
the paper calls current chunk id / aborted primitive id.  Connectors are bounded
FIFOs of K slots with monotone head/tail counters per (collective, ring edge); a
primitive touches nothing until BOTH its conditions hold, so an aborted wait leaves
connectors and buffers unchanged (Sec. 4.5: restart without under- or re-sending).
A preempted collective keeps its queue position (Sec. 4.3).

Readings taken where the paper is silent: spin threshold unit
= poll attempts; thr(pos) = max(spin_min, spin_init >> pos); after a success
thr = min(spin_max, thr*boost) until preemption or completion; "cannot progress for
a while" = one whole pass over the task queue with no successful primitive, after
which up to `fetch_batch` SQEs are fetched (the paper does not say how many).

One tick of a rank = its local bookkeeping up to and including ONE poll attempt,
plus the slice's data movement when the poll succeeds.  Which actor ticks next is
chosen from outside (round-robin, seeded random, or exhaustive search), which is
what lets tests explore interleavings.  Host submitters are actors too.

Slices carry real numpy data, so the model's final buffers can be compared with the
data oracle bit for bit; they also carry (round, step) tags that the receiver checks.

Two variations of Alg. 1 can be switched on, to ask whether they keep its liveness:

  * `lookahead = n > 0`: a successful poll only CLAIMS the slots (the daemon's own view of
    its connector counters advances) and queues the slice; a separate mover actor per rank
    moves queued slices in order and only then are the shared counters raised; at most n
    slices of a rank are claimed and not yet moved.  The wait conditions are evaluated on
    the claimed view: readable = tail - head - (claimed pops) > 0, writable = tail +
    (claimed pushes) - head < K.  A collective whose last slice is claimed leaves the task
    queue at once; its CQE is written when that slice has been moved.
  * `scan = True`: a pass starts by evaluating the wait conditions of every queue entry and
    visits only the entries found runnable, each with the minimum threshold.
  * `direct = True`: the gather steps of an all-reduce (and all steps of an all-gather or a
    broadcast) go without FIFO slots.  A rank writes a
    finished chunk to its recv buffer only and notifies the next rank (the connector's counter is
    raised, no slot is needed, so no wait for space); the next rank copies it out of that recv
    buffer; a last step (drain) waits until the next rank has consumed everything, because
    the buffers belong to the caller again once the completion is posted.  The opening send of
    an all-reduce, a reduce-scatter or a reduce chain moves nothing either: it only notifies, and
    the next rank's first reduce step reads the chunk from this rank's send buffer.
  * `focus = n > 0` (with scan): the runnable entries are visited furthest-along first
    (most primitives done; ties in queue order), and once n slices have been taken in the
    pass it ends with the entry in hand: every rank ranks the collectives alike, so the
    ranks settle on the same few of them (the coalescing of choices that Sec. 4.3 aims at).
  * `fold = True`: collectives run in steps that each wait on ALL ranks (see below for the kinds other than the
    all-reduce); an all-reduce runs in two steps that each wait on ALL ranks instead of 2R-1 steps that
    each wait on the neighbour (every rank's buffers are readable and writable by every other): "fold_scatter"
    waits until every rank has fetched (published) the invocation, then rank r combines chunk r out of all R
    send buffers in the ring's order x[r+1] (op) ... (op) x[r] and writes the result into chunk r of ALL R recv
    buffers; "last_wait_red" waits until every rank has done so (then every chunk of the own recv buffer has
    arrived and nobody reads the own send buffer any more) and moves nothing.  Shared counters per collective
    (published / folded / gathered) carry the waits; each step is still poll-then-move, so a stuck one is
    preempted like any primitive.
    Reduce-scatter: "fold_all" (block r into the own recv buffer), "last_wait_red" (every rank has folded: the
    send buffers are free).  Reduce: "fold_root" (rank r combines chunk r of the message in the chain's order
    x[root+1] (op) ... (op) x[root] into the ROOT's recv buffer), "last_wait_red".  All-gather and broadcast:
    "gather_pub" (once every rank has published: all R blocks out of the send buffers / the root's send
    buffer), "last_wait".
  * `priority_order = True` (Sec. 4.3 "Priority-based Ordering"): the SQ is looked at before every
    pass, a fetched collective is inserted behind the queued ones of equal or higher user priority
    (Coll.priority, larger = more urgent), and a focused pass ranks the runnable entries by
    priority first, progress and queue position only among equals.
"""
from __future__ import annotations

import copy
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import ring_data as rd

AR, AG, RS, BC, RD = 0, 1, 2, 3, 4
CHAINS = (BC, RD)     # one primitive per slice, which one depends on the rank's place in the chain
INF = 1 << 60

# primitive name -> (needs recv, send side), send side: 0 none, 1 waits for a free slot and fills it,
# 2 notify (the result stays in the rank's recv buffer, the counter is raised without a slot),
# 3 drain (no data: waits until the next rank has consumed everything sent or notified so far)
PRIMS = {
    "send": (False, 1),
    "copy_send": (False, 1),
    "copy": (False, 0),
    "recv_reduce_send": (True, 1),
    "recv_reduce_copy_send": (True, 1),
    "recv_reduce_copy": (True, 0),
    "recv_copy_send": (True, 1),
    "recv_copy": (True, 0),
    # direct gather steps of an all-reduce (Policy.direct)
    "recv_reduce_copy_notify": (True, 2),
    "direct_copy_notify": (True, 2),
    "direct_copy": (True, 0),
    "copy_notify": (False, 2),
    "notify": (False, 2),                      # nothing moved: the next rank reads this rank's send buffer
    "direct_reduce_send": (True, 1),           # recv-reduce-send whose input is the previous rank's send buffer
    "direct_reduce_copy_notify": (True, 2),    # the same as the last reduce step (two ranks)
    "direct_reduce_copy": (True, 0),           # the same as the last step of a reduce-scatter (two ranks)
    "drain": (False, 3),
    # fold steps of an all-reduce (Policy.fold): send side 4 / 5 / 6 = wait until every rank has published /
    # folded / gathered this invocation (a shared counter reaches (invocation + 1) x R)
    "fold_all": (False, 4),
    "fold_scatter": (False, 4),     # all-reduce: chunk r combined and written into every rank's recv buffer
    "last_wait": (False, 6),
    "fold_root": (False, 4),        # reduce: chunk r into the root's recv buffer
    "gather_pub": (False, 4),       # all-gather, broadcast: copies out of send buffers once everybody has published
    "last_wait_red": (False, 5),    # reduce-scatter, reduce: every rank has folded
}


@dataclass
class Policy:
    spin_init: int = 8
    spin_min: int = 1
    spin_max: int = 64
    boost: int = 4
    preempt: bool = True
    taskq_cap: int = 1 << 20
    sq_depth: int = 1 << 20
    K: int = 2                    # slots per connector FIFO
    slice_elems: int = 1 << 30    # elements per slice (per round)
    fetch_batch: int = 1          # SQEs fetched in a row when the queue is empty or stuck (0 = all available)
    lookahead: int = 0            # 0: a slice moves at its successful poll; n: up to n claimed slices per rank, moved by a mover actor
    scan: bool = False            # a pass visits only the entries whose wait conditions hold at its start
    focus: int = 0                # with scan: furthest-along entries first, and the pass ends after this many slices
    direct: bool = False          # steps that read the previous rank's recv / send buffer instead of a slot (notify / drain)
    fold: bool = False            # collectives in steps that wait on all ranks (all-reduce: fold_scatter, last_wait_red)
    fold_slice: int = 0           # with fold: elements per slice of the step with data (0 = the whole chunk at once); the
                                  # step is taken slice after slice, the last wait once, behind the last slice
    priority_order: bool = False  # priority-based ordering: fetch before every pass, queue sorted by Coll.priority, priority ranks first


@dataclass
class Coll:
    kind: int
    dtype: int
    count: int
    root: int = 0
    priority: int = 0             # larger = more urgent; used only under Policy.priority_order


def program(kind: int, R: int, r: int, root: int, blocks: List[Tuple[int, int]],
            recv_blocks: List[Tuple[int, int]], direct: bool = False, fold: bool = False):
    """Per-rank primitive sequence: list of (name, send-buffer block, recv-buffer block).
    `blocks` / `recv_blocks` are the element ranges of ring chunk j in the send / recv buffer."""
    none = None
    if R == 1:
        return [("copy", blocks[0], recv_blocks[0])]
    b = lambda j: blocks[j % R]
    d = lambda j: recv_blocks[j % R]
    if kind == AR and fold:
        return [("fold_scatter", b(r), d(r)), ("last_wait_red", none, none)]
    if kind == RS and fold:
        return [("fold_all", b(r), recv_blocks[0]), ("last_wait_red", none, none)]
    if kind == RD and fold:
        return [("fold_root", none, none), ("last_wait_red", none, none)]
    if kind in (AG, BC) and fold:
        return [("gather_pub", none, none), ("last_wait", none, none)]
    if kind == AR:
        p = [("send", b(r - 1), none)]
        p += [("recv_reduce_send", b(r - 1 - s), none) for s in range(1, R - 1)]
        if direct:
            # the opening send only notifies and the next rank's first reduce step reads the chunk from
            # this rank's send buffer; a finished chunk goes to the recv buffer only and the next rank
            # reads it there; the last step waits until the next rank has read them all (the buffers
            # are the caller's again once the completion is posted)
            p[0] = ("notify", b(r - 1), none)
            if R > 2:
                p[1] = ("direct_reduce_send", b(r - 2), none)
                p += [("recv_reduce_copy_notify", b(r), d(r))]
            else:
                p += [("direct_reduce_copy_notify", b(r), d(r))]
            p += [("direct_copy_notify", none, d(r - j)) for j in range(1, R - 1)]
            p += [("direct_copy", none, d(r + 1))]
            p += [("drain", none, none)]
            return p
        p += [("recv_reduce_copy_send", b(r), d(r))]
        p += [("recv_copy_send", none, d(r - j)) for j in range(1, R - 1)]
        p += [("recv_copy", none, d(r + 1))]
        return p
    if kind == RS and direct:
        # as the reduce phase of the direct all-reduce: the opening send only notifies, the next
        # rank's first reduce step reads the chunk from this rank's send buffer, and the drain keeps
        # the completion (after which the send buffer is the caller's again) behind that read
        p = [("notify", b(r - 1), none)]
        if R > 2:
            p += [("direct_reduce_send", b(r - 2), none)]
            p += [("recv_reduce_send", b(r - 1 - s), none) for s in range(2, R - 1)]
            p += [("recv_reduce_copy", b(r), recv_blocks[0])]
        else:
            p += [("direct_reduce_copy", b(r), recv_blocks[0])]
        p += [("drain", none, none)]
        return p
    if kind == RS:
        p = [("send", b(r - 1), none)]
        p += [("recv_reduce_send", b(r - 1 - s), none) for s in range(1, R - 1)]
        p += [("recv_reduce_copy", b(r), recv_blocks[0])]
        return p
    if kind == AG and direct:
        p = [("copy_notify", blocks[0], d(r))]
        p += [("direct_copy_notify", none, d(r - j)) for j in range(1, R - 1)]
        p += [("direct_copy", none, d(r + 1))]
        p += [("drain", none, none)]
        return p
    if kind == AG:
        p = [("copy_send", blocks[0], d(r))]
        p += [("recv_copy_send", none, d(r - j)) for j in range(1, R - 1)]
        p += [("recv_copy", none, d(r + 1))]
        return p
    if kind == BC and direct:
        # one primitive per slice; the drain is a round of its own after the last slice (see System.rounds)
        pos = (r - root) % R
        if pos == 0:
            return [("copy_notify", blocks[0], recv_blocks[0])]
        if pos == R - 1:
            return [("direct_copy", none, recv_blocks[0])]
        return [("direct_copy_notify", none, recv_blocks[0])]
    if kind == BC:
        pos = (r - root) % R
        if pos == 0:
            return [("copy_send", blocks[0], recv_blocks[0])]
        if pos == R - 1:
            return [("recv_copy", none, recv_blocks[0])]
        return [("recv_copy_send", none, recv_blocks[0])]
    if kind == RD:
        # the reduce phase along the chain root+1 -> root+2 -> ... -> root; with direct steps the
        # first rank only notifies and the second reads the slice out of the first one's send buffer
        pos = (r - root - 1) % R
        if pos == 0:
            return [("notify" if direct else "send", blocks[0], none)]
        first_in = "direct_reduce" if direct and pos == 1 else "recv_reduce"
        if pos == R - 1:
            return [(first_in + "_copy", blocks[0], recv_blocks[0])]
        return [(first_in + "_send", blocks[0], none)]
    raise ValueError(kind)


def layout(c: Coll, R: int):
    """(send blocks, recv blocks, block length used for slicing) for a collective."""
    eb = rd.ELEM_BYTES[c.dtype]
    if c.kind == AR:
        cb = rd.chunk_bounds(c.count, R, eb) if R > 1 else [(0, c.count)]
        return cb, cb, max(hi - lo for lo, hi in cb)
    if c.kind == RS:
        return [(j * c.count, (j + 1) * c.count) for j in range(R)], [(0, c.count)] * R, c.count
    if c.kind == AG:
        return [(0, c.count)] * R, [(j * c.count, (j + 1) * c.count) for j in range(R)], c.count
    return [(0, c.count)] * R, [(0, c.count)] * R, c.count


class Fifo:
    __slots__ = ("K", "head", "tail", "slots")

    def __init__(self, K):
        self.K, self.head, self.tail = K, 0, 0
        self.slots = {}            # position -> entry (a notify is not bounded by K, so not a ring of K)

    def readable(self):
        return self.tail > self.head

    def writable(self):
        return self.tail - self.head < self.K

    def push(self, x, need_slot=True):
        assert self.writable() or not need_slot
        self.slots[self.tail] = x
        self.tail += 1

    def pop(self):
        assert self.readable()
        x = self.slots.pop(self.head)
        self.head += 1
        return x


@dataclass
class Stats:
    preemptions: int = 0
    ctx_loads: int = 0
    ctx_saves: int = 0
    lazy_skips: int = 0
    polls: int = 0
    prims: int = 0
    max_taskq: int = 0
    fetches: int = 0


class Daemon:
    """One rank's daemon: Alg. 1 as an explicit state machine."""

    def __init__(self, sysm: "System", r: int):
        self.S, self.r = sysm, r
        self.sq: List[Tuple[int, int]] = []   # (coll, seq) submitted, not yet fetched
        self.taskq: List[int] = []
        self.pos = 0                          # position in task queue of the pass in flight
        self.in_pass = False
        self.pass_progress = False
        self.loaded: Optional[int] = None     # collective in the active context slot
        self.active = None                    # [round, prim] of the loaded collective
        self.dirty = False                    # progressed since load (lazy save)
        self.saved: Dict[int, List[int]] = {} # context buffer: coll -> [round, prim]
        self.spin = 0
        self.thr = 0
        self.exit = False
        self.cq: List[Tuple[int, int]] = []
        self.seq_of: Dict[int, int] = {}
        self.inv_of: Dict[int, int] = {}     # coll -> how often this rank had fetched it before (the same on every rank)
        self.ninv: Dict[int, int] = {}
        self.jobs: List[tuple] = []            # claimed slices not yet moved (lookahead)
        self.ready: Optional[List[int]] = None # queue positions found runnable by the scan of the pass in flight
        self.rk = 0                            # cursor in self.ready
        self.taken = 0                         # slices taken in the pass in flight
        self.stats = Stats()

    # -- Alg. 1 helpers
    def _thr_init(self, pos):
        P = self.S.policy
        if not P.preempt:
            return INF
        return max(P.spin_min, P.spin_init >> min(pos, 60))

    def _fetch(self):
        P = self.S.policy
        if self.sq and len(self.taskq) < P.taskq_cap:
            coll, seq = self.sq.pop(0)
            self.stats.fetches += 1
            if coll < 0:
                self.exit = True
                return
            if P.priority_order:
                pr = self.S.colls[coll].priority
                at = len(self.taskq)
                while at > 0 and self.S.colls[self.taskq[at - 1]].priority < pr:
                    at -= 1
                self.taskq.insert(at, coll)      # stable: behind the queued ones of equal or higher priority
            else:
                self.taskq.append(coll)
            self.seq_of[coll] = seq
            self.inv_of[coll] = self.ninv.get(coll, 0)
            self.ninv[coll] = self.inv_of[coll] + 1
            self.saved[coll] = [0, 0]
            if self.S.is_fold(coll):
                self.S.foldcnt[coll][0] += 1     # the buffers of this invocation are published at the fetch
            self.stats.max_taskq = max(self.stats.max_taskq, len(self.taskq))

    def _load(self, coll):
        self.loaded = coll
        self.active = list(self.saved[coll])
        self.dirty = False
        self.stats.ctx_loads += 1

    def _save(self):
        if self.dirty:
            self.saved[self.loaded] = list(self.active)
            self.stats.ctx_saves += 1
        else:
            self.stats.lazy_skips += 1
        self.loaded = None

    def idle(self):
        return not self.taskq and not self.sq and not self.jobs

    def _conds(self, coll, p):
        """(readable, writable) of collective `coll`'s primitive p on the claimed view of the connectors."""
        S = self.S
        fin = S.fifo[coll][(self.r - 1) % S.R]
        fout = S.fifo[coll][self.r]
        pops = sum(1 for j in self.jobs if j[0] == coll and PRIMS[j[3]][0])
        pushes = sum(1 for j in self.jobs if j[0] == coll and PRIMS[j[3]][1] in (1, 2))
        return (fin.tail - fin.head - pops > 0, fout.tail + pushes - fout.head < fout.K,
                fout.tail + pushes - fout.head == 0)

    def _done(self, coll):
        """Primitives of the invocation this rank has taken so far."""
        g, p = self.active if self.loaded == coll else self.saved[coll]
        return g * len(self.S.progs[coll][self.r]) + p

    def _next_entry(self, left_queue_at: Optional[int] = None):
        """Scanned pass: go on to the next list entry.  An entry that left the queue moves the
        ones behind it up by one; a focused pass that has taken its share of slices ends here."""
        self.rk += 1
        if left_queue_at is not None:
            self.ready = [i - 1 if (k >= self.rk and i > left_queue_at) else i for k, i in enumerate(self.ready)]
        if self.S.policy.focus and self.taken >= self.S.policy.focus:
            self.rk = len(self.ready)

    def _prim(self, coll, g, p):
        """(name, send block, recv block) of primitive p of round g."""
        S = self.S
        if S.policy.direct and not S.is_fold(coll) and S.colls[coll].kind in CHAINS and S.R > 1 and g == S.rounds[coll] - 1:
            return ("drain", None, None)
        return S.progs[coll][self.r][p]

    def _fold_ok(self, coll, send_side):
        """Fold steps: the shared counter of the step (4 published, 5 folded, 6 gathered) has reached every rank's
        share of this invocation."""
        if send_side < 4:
            return True
        # (published: once per rank and invocation; folded / gathered: once per rank, invocation and slice)
        per_rank = 1 if send_side == 4 else self.S.rounds[coll]
        return self.S.foldcnt[coll][send_side - 4] >= (self.inv_of[coll] + 1) * self.S.R * per_rank

    def _runnable(self, coll):
        g, p = self.active if self.loaded == coll else self.saved[coll]
        need_recv, send_side = PRIMS[self._prim(coll, g, p)[0]]
        rd_ok, wr_ok, drained = self._conds(coll, p)
        return ((not need_recv or rd_ok) and (send_side != 1 or wr_ok) and (send_side != 3 or drained)
                and self._fold_ok(coll, send_side))

    def mover_tick(self) -> bool:
        """Move the oldest claimed slice (lookahead mode): data, shared counters, and the CQE if it was the last."""
        if not self.jobs:
            return False
        coll, g, p, name, sblk, dblk, last = self.jobs.pop(0)
        S = self.S
        S.move(coll, self.r, g, p, name, sblk, dblk, S.fifo[coll][(self.r - 1) % S.R], S.fifo[coll][self.r])
        if last:
            self.cq.append((coll, self.seq_of[coll]))
        return True

    def tick(self) -> bool:
        """Advance to (and perform) one poll attempt. Returns True if the state changed."""
        if self.exit:
            return False
        changed = False
        while True:
            if not self.in_pass:
                # FetchSQE: when the queue is empty, or the last pass made no progress
                before = (len(self.taskq), len(self.sq))
                if not self.taskq or not self.pass_progress or self.S.policy.priority_order:
                    n = self.S.policy.fetch_batch or (1 << 30)
                    while n > 0 and self.sq and not self.exit and len(self.taskq) < self.S.policy.taskq_cap:
                        self._fetch()
                        n -= 1
                if self.exit:
                    return True
                if (len(self.taskq), len(self.sq)) != before:
                    changed = True
                if not self.taskq:
                    return changed
                self.in_pass, self.pos, self.pass_progress = True, 0, False
                if self.S.policy.scan:
                    self.ready = [i for i, c in enumerate(self.taskq) if self._runnable(c)]
                    if self.S.policy.focus and self.S.policy.priority_order:
                        self.ready.sort(key=lambda i: (-self.S.colls[self.taskq[i]].priority, -self._done(self.taskq[i]), i))
                    elif self.S.policy.focus:
                        self.ready.sort(key=lambda i: (-self._done(self.taskq[i]), i))
                    self.rk, self.taken = 0, 0
                    if not self.ready:
                        self.in_pass = False   # nothing can run: the pass is over before it began
                        if self.loaded is not None:
                            self._save()
                            changed = True
                        return changed
            if self.S.policy.scan:
                self.pos = self.ready[self.rk] if self.rk < len(self.ready) else len(self.taskq)
            if self.pos >= len(self.taskq):
                self.in_pass = False
                if self.loaded is not None:
                    self._save()
                # a pass ended; a new pass (and maybe a fetch) starts at the next tick
                return True
            coll = self.taskq[self.pos]
            if self.loaded != coll:
                if self.loaded is not None:
                    self._save()
                self._load(coll)
                self.thr = self._thr_init(self.pos)
                if self.S.policy.scan and self.S.policy.preempt:
                    self.thr = self.S.policy.spin_min
                self.spin = 0
                changed = True
            return self._poll_and_run(coll) or changed

    def _poll_and_run(self, coll) -> bool:
        S = self.S
        P = S.policy
        rounds, prog = S.rounds[coll], S.progs[coll][self.r]
        g, p = self.active
        name, sblk, dblk = self._prim(coll, g, p)
        need_recv, send_side = PRIMS[name]
        fin = S.fifo[coll][(self.r - 1) % S.R]
        fout = S.fifo[coll][self.r]
        self.stats.polls += 1
        rd_ok, wr_ok, drained = self._conds(coll, p)
        ok = ((not need_recv or rd_ok) and (send_side != 1 or wr_ok) and (send_side != 3 or drained)
              and self._fold_ok(coll, send_side))
        if not ok:
            if self.thr >= INF:
                return False               # spins forever: no state change
            self.spin += 1
            if self.spin >= self.thr:
                self.stats.preemptions += 1
                self._save()
                if P.scan:
                    self._next_entry()
                else:
                    self.pos += 1
            return True
        if P.lookahead and len(self.jobs) >= P.lookahead:
            return False                   # every claim slot is taken: wait for the mover (no state change)
        # ---- the slice is this rank's now: moved at once, or claimed and queued for the mover
        p2, g2 = p + 1, g
        if S.is_fold(coll) and len(prog) == 2:
            # fold steps: the step with data for every slice, then the last wait once
            if p == 0:
                p2, g2 = (0, g + 1) if g + 1 < rounds else (1, g)
            else:
                p2, g2 = 0, rounds
        elif p2 == len(prog):
            p2, g2 = 0, g + 1
        last = g2 == rounds
        if P.lookahead:
            self.jobs.append((coll, g, p, name, sblk, dblk, last))
        else:
            S.move(coll, self.r, g, p, name, sblk, dblk, fin, fout)
        self.stats.prims += 1
        self.taken += 1
        self.dirty = True
        self.pass_progress = True
        self.spin = 0
        if P.preempt and not P.scan:
            self.thr = min(P.spin_max, self.thr * P.boost)
        self.active = [g2, p2]
        if last:
            # CollectiveSuccess -> SendCQE; entry leaves the queue, position stays
            if not P.lookahead:
                self.cq.append((coll, self.seq_of[coll]))
            self.taskq.pop(self.pos)
            self.saved[coll] = [0, 0]
            self.loaded = None
            if P.scan:
                self._next_entry(left_queue_at=self.pos)
        return True


class System:
    def __init__(self, R: int, colls: Sequence[Coll], sends: Optional[List[List[np.ndarray]]],
                 policy: Policy):
        """sends[ci][r] = rank r's send buffer for collective ci (None -> tokens only)."""
        self.R, self.colls, self.policy = R, list(colls), policy
        self.with_data = sends is not None
        self.sends = sends
        self.recvs = None
        if self.with_data:
            self.recvs = []
            for ci, c in enumerate(colls):
                n = c.count * R if c.kind == AG else c.count
                self.recvs.append([np.zeros(n, dtype=sends[ci][0].dtype) for _ in range(R)])
        self.progs, self.rounds, self.fifo = [], [], []
        for c in colls:
            sb, db, blen = layout(c, R)
            is_fold = policy.fold and R > 1
            self.progs.append([program(c.kind, R, r, c.root, sb, db, policy.direct, is_fold) for r in range(R)])
            if is_fold:      # fold steps: one slice per share, or slices of fold_slice elements
                self.rounds.append(max(1, -(-blen // policy.fold_slice)) if policy.fold_slice else 1)
            else:
                self.rounds.append(max(1, -(-blen // policy.slice_elems)))
            if policy.direct and c.kind in CHAINS and R > 1 and not is_fold:
                self.rounds[-1] += 1     # the last round of a chain with direct steps is the drain
            self.fifo.append([Fifo(policy.K) for _ in range(R)])
        self.foldcnt = [[0, 0, 0] for _ in colls]     # fold steps: ranks that have published / folded / gathered, over all invocations
        self.daemons = [Daemon(self, r) for r in range(R)]
        self.pending = [[] for _ in range(R)]   # host side: submissions not yet pushed to the SQ
        self.nsub = [0] * R

    # -- host side
    def plan(self, orders: Sequence[Sequence[int]]):
        for r, o in enumerate(orders):
            self.pending[r] = list(o)

    def host_tick(self, r) -> bool:
        """Host thread of rank r pushes its next submission if the SQ has room."""
        if not self.pending[r] or len(self.daemons[r].sq) >= self.policy.sq_depth:
            return False
        self.daemons[r].sq.append((self.pending[r].pop(0), self.nsub[r]))
        self.nsub[r] += 1
        return True

    def submit_all(self):
        for r in range(self.R):
            while self.host_tick(r):
                pass

    def is_fold(self, ci) -> bool:
        return self.policy.fold and self.R > 1

    # -- data phase
    def _slice(self, blk, g):
        if blk is None:
            return None
        s = self.policy.slice_elems
        lo, hi = blk
        return (min(lo + g * s, hi), min(lo + (g + 1) * s, hi))

    def move(self, ci, r, g, p, name, sblk, dblk, fin, fout):
        c = self.colls[ci]
        tag_out = (g, p)
        x = None
        if name in ("drain", "last_wait", "last_wait_red"):
            return
        if name in ("fold_all", "fold_scatter", "fold_root", "gather_pub"):
            # slice g of the chunk (the whole chunk when there is one slice), read out of the other ranks' buffers in place
            if self.with_data:
                R = self.R
                fs = self.policy.fold_slice

                def cut(blk):
                    lo, hi = blk
                    return (lo, hi) if not fs else (min(lo + g * fs, hi), min(lo + (g + 1) * fs, hi))
                if name == "fold_all":        # reduce-scatter: block r; the ring's order, which begins behind r
                    (slo, shi), (dlo, dhi) = cut(sblk), cut(dblk)
                    self.recvs[ci][r][dlo:dhi] = rd.fold_rotated([s[slo:shi] for s in self.sends[ci]], r + 1, c.dtype)
                elif name == "fold_scatter":  # all-reduce: chunk r in the same order, into every rank's recv buffer
                    (slo, shi), (dlo, dhi) = cut(sblk), cut(dblk)
                    x = rd.fold_rotated([s[slo:shi] for s in self.sends[ci]], r + 1, c.dtype)
                    for j in range(R):
                        self.recvs[ci][j][dlo:dhi] = x
                elif name == "fold_root":     # reduce: chunk r of the message, the chain's order, into the root's buffer
                    lo, hi = cut(rd.chunk_bounds(c.count, R, rd.ELEM_BYTES[c.dtype])[r])
                    self.recvs[ci][c.root][lo:hi] = rd.fold_rotated([s[lo:hi] for s in self.sends[ci]], c.root + 1, c.dtype)
                elif c.kind == AG:            # all-gather: block j out of rank j's send buffer
                    lo, hi = cut((0, c.count))
                    for j in range(R):
                        self.recvs[ci][r][j * c.count + lo:j * c.count + hi] = self.sends[ci][j][lo:hi]
                else:                         # broadcast: the root's send buffer
                    lo, hi = cut((0, c.count))
                    self.recvs[ci][r][lo:hi] = self.sends[ci][c.root][lo:hi]
            self.foldcnt[ci][1 if name.startswith("fold") else 2] += 1
            return
        if PRIMS[name][0]:
            tag, x = fin.pop()
            # the sender's primitive index of this hop is p-1 in every ring sequence here,
            # except the chains (broadcast, reduce) where every rank has a one-primitive program
            want = (g, 0) if c.kind in CHAINS else (g, p - 1)
            assert tag == want, f"slice out of sequence: got {tag}, want {want}"
        if self.with_data:
            ss, ds = self._slice(sblk, g), self._slice(dblk, g)
            src = self.sends[ci][r]
            dst = self.recvs[ci][r]
            if isinstance(x, tuple):
                # a notified chunk: read now from the buffer of the rank that holds it
                if x[0] == "direct_send":
                    x = self.sends[ci][x[1]][ss[0]:ss[1]].copy()     # same chunk, same offsets in its send buffer
                else:
                    x = self.recvs[ci][x[1]][ds[0]:ds[1]].copy()
            if name == "notify":
                y = None
            elif name in ("send", "copy_send", "copy", "copy_notify"):
                y = src[ss[0]:ss[1]].copy()
            elif name.startswith("direct_reduce"):
                y = rd.add_hop(x, src[ss[0]:ss[1]], c.dtype)
            elif name.startswith("recv_reduce"):
                y = rd.add_hop(x, src[ss[0]:ss[1]], c.dtype)
            else:
                y = x
            if "copy" in name:
                dst[ds[0]:ds[1]] = y
        else:
            y = None
        if PRIMS[name][1] == 1:
            fout.push((tag_out, y))
        elif PRIMS[name][1] == 2:
            tok = ("direct_send", r) if name == "notify" else ("direct", r)
            fout.push((tag_out, tok if self.with_data else None), need_slot=False)

    # -- global predicates
    def done(self):
        return all(not d.taskq and not d.sq and not d.jobs for d in self.daemons) and not any(self.pending)

    def total_cqes(self):
        return sum(len(d.cq) for d in self.daemons)

    def key(self):
        """Hashable control state (data excluded: it is a function of the counters)."""
        ds = []
        for d in self.daemons:
            ds.append((tuple(d.sq), tuple(d.taskq), d.pos, d.in_pass, d.pass_progress, d.loaded,
                       tuple(d.active) if d.active and d.loaded is not None else None, d.dirty,
                       tuple(sorted((k, tuple(v)) for k, v in d.saved.items())), d.spin, d.thr, len(d.cq),
                       tuple((j[0], j[1], j[2]) for j in d.jobs),
                       (tuple(d.ready), d.rk, d.taken if self.policy.focus else 0) if d.in_pass and d.ready is not None else None))
        fs = tuple((f.head, f.tail) for fl in self.fifo for f in fl)
        return (tuple(ds), fs, tuple(tuple(p) for p in self.pending), tuple(tuple(c) for c in self.foldcnt))

    def clone(self):
        """Copy of the token-only model (immutable program tables are shared)."""
        assert not self.with_data, "clone only the token-only model"
        T = System.__new__(System)
        T.R, T.colls, T.policy = self.R, self.colls, self.policy
        T.with_data, T.sends, T.recvs = False, None, None
        T.progs, T.rounds = self.progs, self.rounds
        T.foldcnt = [list(c) for c in self.foldcnt]
        T.fifo = []
        for fl in self.fifo:
            row = []
            for f in fl:
                g = Fifo(f.K)
                g.head, g.tail, g.slots = f.head, f.tail, dict(f.slots)
                row.append(g)
            T.fifo.append(row)
        T.daemons = []
        for d in self.daemons:
            e = Daemon.__new__(Daemon)
            e.S, e.r = T, d.r
            e.sq, e.taskq = list(d.sq), list(d.taskq)
            e.pos, e.in_pass, e.pass_progress = d.pos, d.in_pass, d.pass_progress
            e.loaded, e.dirty = d.loaded, d.dirty
            e.active = list(d.active) if d.active is not None else None
            e.saved = {k: list(v) for k, v in d.saved.items()}
            e.spin, e.thr, e.exit = d.spin, d.thr, d.exit
            e.cq, e.seq_of = list(d.cq), dict(d.seq_of)
            e.inv_of, e.ninv = dict(d.inv_of), dict(d.ninv)
            e.jobs = list(d.jobs)
            e.ready = list(d.ready) if d.ready is not None else None
            e.rk, e.taken = d.rk, d.taken
            e.stats = copy.copy(d.stats)
            T.daemons.append(e)
        T.pending = [list(p) for p in self.pending]
        T.nsub = list(self.nsub)
        return T


# ----------------------------------------------------------------------------
# choosers
# ----------------------------------------------------------------------------
def run_round_robin(S: System, max_ticks: int = 10_000_000) -> int:
    """Fair chooser. Returns ticks used; raises TimeoutError at the watchdog."""
    t = 0
    while not S.done():
        for r in range(S.R):
            S.host_tick(r)
            S.daemons[r].tick()
            S.daemons[r].mover_tick()
            t += 1
        if t > max_ticks:
            raise TimeoutError("tick watchdog")
    return t


def run_random(S: System, seed: int, max_ticks: int = 10_000_000, host_weight: float = 0.2) -> int:
    """Seeded random chooser over daemons and host submitters (fair with probability 1)."""
    g = np.random.default_rng(seed)
    t = 0
    R = S.R
    while not S.done():
        # draw a batch of choices at once
        for a in g.integers(0, 3 * R, size=256):
            a = int(a)
            if a >= 2 * R:
                S.daemons[a - 2 * R].mover_tick()
            elif a >= R:
                if g.random() < host_weight * 2:
                    S.host_tick(a - R)
            else:
                S.daemons[a].tick()
            t += 1
        if t > max_ticks:
            raise TimeoutError("tick watchdog")
    return t


def is_deadlocked(S: System) -> bool:
    """True if work is outstanding and no actor's tick changes the control state."""
    if S.done():
        return False
    k0 = S.key()
    T = S.clone()
    for r in range(T.R):
        T.host_tick(r)
        T.daemons[r].tick()
        T.daemons[r].mover_tick()
    return T.key() == k0


def explore(S0: System, max_states: int = 2_000_000):
    """Exhaustive search over all interleavings of daemon ticks (token-only model).
    Returns (number of states, list of reachable keys -> a representative System)."""
    assert not S0.with_data
    seen = {S0.key(): S0}
    stack = [S0]
    while stack:
        S = stack.pop()
        for a in range(3 * S.R):
            T = S.clone()
            if a >= 2 * S.R:
                moved = T.daemons[a - 2 * S.R].mover_tick()
            elif a >= S.R:
                moved = T.host_tick(a - S.R)
            else:
                moved = T.daemons[a].tick()
            if not moved:
                continue
            k = T.key()
            if k not in seen:
                seen[k] = T
                stack.append(T)
                if len(seen) > max_states:
                    raise MemoryError("state bound exceeded")
    return seen
