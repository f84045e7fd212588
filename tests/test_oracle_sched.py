"""Pins for the scheduler model (oracle/sched_model.py): liveness under deadlock-prone
issue orders, the no-preemption negative control, and preemption transparency (the data an
interleaved, preempted execution produces equals the data oracle's, bit for bit)."""
import itertools

import numpy as np
import pytest

import workload_inputs as wi
from oracle import ring_data as rd
from oracle import sched_model as sm


def _system(w: wi.Workload, policy: sm.Policy, data=True, priorities=None):
    colls = [sm.Coll(c.kind, c.dtype, c.count, c.root, 0 if priorities is None else priorities[i]) for i, c in enumerate(w.colls)]
    sends = [wi.all_sends(w, ci) for ci in range(len(w.colls))] if data else None
    S = sm.System(w.R, colls, sends, policy)
    S.plan(w.orders)
    return S


def _check_data(S, w):
    for ci, c in enumerate(w.colls):
        want = rd.run_closed_form(c.kind, S.sends[ci], c.dtype, c.root)
        for r in range(w.R):
            assert np.array_equal(S.recvs[ci][r].view(np.uint8), want[r].view(np.uint8)), (ci, r)


ORDERS2 = list(itertools.product([(0, 1), (1, 0)], repeat=2))


@pytest.mark.parametrize("orders", ORDERS2)
@pytest.mark.parametrize("K,slice_elems,spin", [(2, 256, 2), (2, 128, 3), (3, 64, 1), (4, 1024, 8)])
def test_config1_all_issue_orders_complete_and_match(orders, K, slice_elems, spin):
    w = wi.config1(*orders)
    S = _system(w, sm.Policy(spin_init=spin, spin_min=1, spin_max=4 * spin, boost=2, K=K, slice_elems=slice_elems))
    sm.run_round_robin(S, max_ticks=200_000)
    assert S.total_cqes() == 4
    _check_data(S, w)
    # values are small integers: exact sums regardless of order
    for ci in range(2):
        exact = sum(s.astype(np.int64) for s in S.sends[ci])
        for r in range(2):
            assert np.array_equal(S.recvs[ci][r].astype(np.int64), exact)


@pytest.mark.parametrize("seed", range(6))
def test_config1_random_interleavings(seed):
    w = wi.config1((0, 1), (1, 0))
    S = _system(w, sm.Policy(spin_init=3, spin_max=12, boost=2, K=2, slice_elems=128))
    sm.run_random(S, seed, max_ticks=500_000)
    _check_data(S, w)
    assert sum(d.stats.preemptions for d in S.daemons) > 0


def test_negative_control_without_preemption_deadlocks():
    """Opposite issue orders + no preemption = the single-queue deadlock of Sec. 2.3 / Fig. 1(c);
    the paper reports a 100 % deadlock ratio for the non-preemptive library (Sec. 6.1)."""
    w = wi.config1((0, 1), (1, 0))
    S = _system(w, sm.Policy(preempt=False, K=2, slice_elems=256, taskq_cap=1), data=False)
    S.submit_all()
    with pytest.raises(TimeoutError):
        sm.run_round_robin(S, max_ticks=5_000)
    assert sm.is_deadlocked(S)
    assert S.total_cqes() == 0


def test_same_order_without_preemption_completes():
    w = wi.config1((0, 1), (0, 1))
    S = _system(w, sm.Policy(preempt=False, K=2, slice_elems=256, taskq_cap=1))
    sm.run_round_robin(S, max_ticks=100_000)
    _check_data(S, w)
    assert not sm.is_deadlocked(S)


@pytest.mark.parametrize("orders", ORDERS2)
@pytest.mark.parametrize("K", [2, 3])
def test_exhaustive_interleavings_tiny(orders, K):
    """2 ranks, 2 collectives, 2 slices each, K slots: every reachable control state (all
    interleavings of daemon ticks and host submissions) can still finish under a fair chooser,
    and no reachable state is a deadlock."""
    w = wi.config1(*orders, n=8)
    pol = sm.Policy(spin_init=2, spin_min=1, spin_max=2, boost=2, K=K, slice_elems=2)
    S0 = _system(w, pol, data=False)
    seen = sm.explore(S0, max_states=400_000)
    assert len(seen) > 100
    finals = 0
    # every 17th state (plus all states when the space is small) is driven to completion
    keys = list(seen)
    step = 1 if len(keys) < 3000 else 17
    for k in keys[::step]:
        T = seen[k].clone()
        assert not sm.is_deadlocked(T)
        sm.run_round_robin(T, max_ticks=50_000)
        assert T.total_cqes() == 4
        finals += 1
    assert finals > 0


def test_R3_three_collectives_all_216_orders():
    R = 3
    colls = [wi.CollSpec(i, wi.AR, wi.F32, 48) for i in range(3)]
    perms = list(itertools.permutations(range(3)))
    for o0, o1, o2 in itertools.product(perms, repeat=3):
        w = wi.Workload("r3", R, colls, [list(o0), list(o1), list(o2)], seed=5, cfg=90)
        S = _system(w, sm.Policy(spin_init=4, spin_max=16, boost=2, K=2, slice_elems=8), data=False)
        sm.run_round_robin(S, max_ticks=200_000)
        assert S.total_cqes() == 9


@pytest.mark.parametrize("seed", range(3))
def test_mixed_kinds_preemption_transparent(seed):
    """All four kinds, three dtypes, uneven sizes, random per-rank orders, tiny thresholds:
    thousands of preemptions, results identical to the data oracle."""
    w = wi.config4(n_colls=10, min_bytes=256, max_bytes=4096, seed=seed, R=4)
    S = _system(w, sm.Policy(spin_init=4, spin_min=1, spin_max=16, boost=2, K=2, slice_elems=40, sq_depth=3))
    sm.run_random(S, seed + 100, max_ticks=5_000_000)
    assert S.total_cqes() == 10 * 4
    _check_data(S, w)
    assert sum(d.stats.preemptions for d in S.daemons) > 50
    assert sum(d.stats.lazy_skips for d in S.daemons) > 0


def test_uneven_allreduce_bf16_through_scheduler():
    R = 5
    colls = [wi.CollSpec(0, wi.AR, wi.BF16, 131), wi.CollSpec(1, wi.AR, wi.F16, 7), wi.CollSpec(2, wi.AR, wi.I32, 3)]
    orders = [list(np.random.default_rng(r).permutation(3)) for r in range(R)]
    w = wi.Workload("uneven", R, colls, orders, seed=9, cfg=91)
    S = _system(w, sm.Policy(spin_init=2, spin_max=8, boost=2, K=2, slice_elems=8))
    sm.run_round_robin(S, max_ticks=1_000_000)
    _check_data(S, w)


def test_stickiness_thresholds_follow_position_and_boost():
    w = wi.config1((0, 1), (0, 1))
    pol = sm.Policy(spin_init=64, spin_min=4, spin_max=1000, boost=20)
    S = _system(w, pol, data=False)
    d = S.daemons[0]
    assert [d._thr_init(p) for p in range(6)] == [64, 32, 16, 8, 4, 4]
    S.submit_all()
    d.tick()                       # loads collective 0 and runs its first primitive (send: always possible)
    assert d.thr == min(1000, 64 * 20)
    assert d.stats.prims == 1


def test_task_queue_capacity_is_a_liveness_condition():
    """With preemption on but a one-entry task queue, opposite orders still deadlock: the peer's
    collective can never be fetched. Capacity >= outstanding collectives restores liveness."""
    w = wi.config1((0, 1), (1, 0))
    S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=256, taskq_cap=1), data=False)
    with pytest.raises(TimeoutError):
        sm.run_round_robin(S, max_ticks=20_000)
    assert S.total_cqes() == 0
    S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=256, taskq_cap=2), data=False)
    sm.run_round_robin(S, max_ticks=20_000)
    assert S.total_cqes() == 4


def test_one_slot_connectors_cannot_run_a_fused_ring():
    """K = 1 is not a valid connector depth: after every rank's opening `send` all connectors are
    full and every next primitive needs its send side writable AND its recv side readable, so even
    a single collective in a consistent order stalls. The library therefore requires K >= 2."""
    w = wi.config1((0, 1), (0, 1))
    S = _system(w, sm.Policy(spin_init=2, spin_max=8, boost=2, K=1, slice_elems=256), data=False)
    with pytest.raises(TimeoutError):
        sm.run_round_robin(S, max_ticks=20_000)
    assert S.total_cqes() == 0


@pytest.mark.parametrize("batch", [0, 3])
def test_batch_fetch_keeps_liveness_and_values(batch):
    """Fetching several SQEs at once when stuck (the GPU path's default) changes timing only."""
    w = wi.config4(n_colls=8, min_bytes=256, max_bytes=2048, seed=11, R=3)
    S = _system(w, sm.Policy(spin_init=3, spin_min=1, spin_max=12, boost=2, K=2, slice_elems=32, fetch_batch=batch))
    sm.run_random(S, 5, max_ticks=5_000_000)
    assert S.total_cqes() == 8 * 3
    _check_data(S, w)


# ---------------------------------------------------------------- claim-ahead and scan variations
VARIANTS = [dict(lookahead=1), dict(lookahead=2), dict(scan=True), dict(lookahead=2, scan=True),
            dict(scan=True, focus=1), dict(lookahead=2, scan=True, focus=2),
            dict(direct=True), dict(lookahead=2, scan=True, focus=1, direct=True)]


@pytest.mark.parametrize("var", [dict(lookahead=2), dict(scan=True), dict(lookahead=2, scan=True),
                                 dict(lookahead=2, scan=True, focus=1), dict(direct=True),
                                 dict(lookahead=2, scan=True, direct=True)])
@pytest.mark.parametrize("orders", [((0, 1), (1, 0)), ((0, 1), (0, 1))])
def test_variations_exhaustive_interleavings_tiny(orders, var):
    """Claiming slices ahead of their movement (a mover actor raises the shared counters later),
    visiting only runnable entries, and visiting them furthest-along first in passes that end after a
    fixed number of slices, and direct gather steps (notify without a slot, drain before completion)
    keep Alg. 1's liveness: in the circular-wait setting no reachable
    state -- over all interleavings of daemons, movers and host submissions -- is a deadlock, and every
    one of them finishes with all four CQEs."""
    # (without the scan the state space is large: one slice per collective there, two with it)
    w = wi.config1(*orders, n=8)
    pol = sm.Policy(spin_init=2, spin_min=1, spin_max=2, boost=2, K=2, slice_elems=2 if var.get("scan") else 4, **var)
    S0 = _system(w, pol, data=False)
    seen = sm.explore(S0, max_states=600_000)
    assert len(seen) > 20
    keys = list(seen)
    step = 1 if len(keys) < 1000 else 97
    for k in keys[::step]:
        T = seen[k].clone()
        assert not sm.is_deadlocked(T)
        sm.run_round_robin(T, max_ticks=50_000)
        assert T.total_cqes() == 4


@pytest.mark.parametrize("var", VARIANTS)
@pytest.mark.parametrize("seed", range(3))
def test_variations_are_transparent_to_the_values(var, seed):
    """Mixed kinds on three ranks, random issue orders, random interleavings of daemons, movers and
    hosts: with slices claimed ahead / runnable-only passes the final buffers equal the data oracle's."""
    g = np.random.default_rng(seed)
    R = 3
    colls = [wi.CollSpec(0, wi.AR, wi.F32, 50), wi.CollSpec(1, wi.AG, wi.F16, 12),
             wi.CollSpec(2, wi.RS, wi.I32, 16), wi.CollSpec(3, wi.BC, wi.BF16, 40, root=2),
             wi.CollSpec(4, wi.AR, wi.BF16, 33)]
    orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]
    w = wi.Workload("var", R, colls, orders, seed=seed, cfg=91)
    S = _system(w, sm.Policy(spin_init=3, spin_max=6, boost=2, K=2, slice_elems=8, **var))
    sm.run_random(S, seed + 100, max_ticks=2_000_000)
    assert S.total_cqes() == R * len(colls)
    _check_data(S, w)


def test_claims_never_overrun_a_connector():
    """With two claims allowed and two-slot connectors the claimed view keeps every FIFO within its
    capacity at every tick, and a collective's CQE never precedes the movement of its last slice."""
    w = wi.config1((0, 1), (1, 0), n=64)
    S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=4, lookahead=2))
    g = np.random.default_rng(3)
    ticks = 0
    while not S.done():
        a = int(g.integers(0, 6))
        if a >= 4:
            S.daemons[a - 4].mover_tick()
        elif a >= 2:
            S.host_tick(a - 2)
        else:
            S.daemons[a].tick()
        for fl in S.fifo:
            for f in fl:
                assert 0 <= f.tail - f.head <= f.K
        for d in S.daemons:
            assert len(d.jobs) <= 2
            done_colls = {c for c, _ in d.cq}
            assert not any(j[0] in done_colls for j in d.jobs)
        ticks += 1
        assert ticks < 1_000_000
    assert S.total_cqes() == 4
    _check_data(S, w)


def test_negative_control_still_deadlocks_with_claims():
    """Claim-ahead does not hide the need for preemption: opposite orders without it still deadlock."""
    w = wi.config1((0, 1), (1, 0))
    S = _system(w, sm.Policy(preempt=False, K=2, slice_elems=256, taskq_cap=1, lookahead=2), data=False)
    with pytest.raises(TimeoutError):
        sm.run_round_robin(S, max_ticks=20_000)
    assert sm.is_deadlocked(S)


def test_focused_passes_take_the_furthest_along_first():
    """focus = 1: after the scan of a pass the daemon works on the runnable collective with the most
    primitives done (ties: queue order), and the pass ends with that entry."""
    colls = [wi.CollSpec(i, wi.AR, wi.I32, 24) for i in range(3)]
    w = wi.Workload("focus", 2, colls, [[0, 1, 2], [0, 1, 2]], seed=4, cfg=92)
    S = _system(w, sm.Policy(spin_init=1, spin_min=1, spin_max=1, boost=1, K=2, slice_elems=4, scan=True, focus=1, fetch_batch=0))
    for r in range(2):
        while S.pending[r]:
            S.host_tick(r)
    d0, d1 = S.daemons
    picks = []
    for _ in range(400):
        if S.done():
            break
        for d in (d0, d1):
            was = d.in_pass
            d.tick()
            if d is d0 and d.in_pass and not was and d.ready:
                # a pass has just begun: its list is sorted by primitives done, then queue position
                done = [d._done(d.taskq[i]) for i in d.ready]
                assert done == sorted(done, reverse=True)
                assert all(a < b for a, b, x, y in zip(d.ready, d.ready[1:], done, done[1:]) if x == y)
                picks.append(d.taskq[d.ready[0]])
    assert S.done() and S.total_cqes() == 6
    _check_data(S, w)
    # the first collective is carried through before the last one is begun
    assert picks.index(2) > max(i for i, c in enumerate(picks) if c == 0) - 2


def test_direct_gather_steps_wait_for_the_reader_before_completing():
    """direct = True: a rank's completion is posted only after the next rank has copied every notified
    chunk out of its recv buffer (drain), whatever the interleaving; the values equal the data oracle's
    and no FIFO slot is ever used by a gather step (the connectors never hold more than K slot entries,
    notifications aside)."""
    R = 3
    colls = [wi.CollSpec(0, wi.AR, wi.F32, 50), wi.CollSpec(1, wi.AR, wi.BF16, 33), wi.CollSpec(2, wi.AR, wi.I32, 7)]
    for seed in range(4):
        g = np.random.default_rng(seed)
        orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]
        w = wi.Workload("direct", R, colls, orders, seed=seed, cfg=93)
        S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=8, direct=True, lookahead=2))
        assert [p[0] for p in S.progs[0][0]][-4:] == ["recv_reduce_copy_notify", "direct_copy_notify", "direct_copy", "drain"]
        assert [p[0] for p in sm.program(wi.AG, 4, 1, 0, [(0, 8)], [(8 * j, 8 * j + 8) for j in range(4)], True)] == \
            ["copy_notify", "direct_copy_notify", "direct_copy_notify", "direct_copy", "drain"]
        posted = {}
        rng = np.random.default_rng(100 + seed)
        for _ in range(2_000_000):
            if S.done():
                break
            a = int(rng.integers(0, 3 * R))
            r = a % R
            if a < R:
                S.host_tick(r)
            elif a < 2 * R:
                S.daemons[r].mover_tick()
            else:
                S.daemons[r].tick()
            for d in S.daemons:
                for (c, seq) in d.cq:
                    if (d.r, c) not in posted:
                        posted[(d.r, c)] = True
                        f = S.fifo[c][d.r]
                        assert f.tail == f.head, "completion posted while the next rank still had chunks to read"
        assert S.done() and S.total_cqes() == R * len(colls)
        _check_data(S, w)


@pytest.mark.parametrize("R", [2, 4])
def test_direct_reduce_scatter_reads_the_send_buffer_and_drains(R):
    """direct = True, reduce-scatter: the opening send moves nothing, the next rank's first reduce step
    takes the block out of this rank's send buffer, and the completion (after which the caller may
    overwrite the send buffer) waits until that read has happened; values as the data oracle's."""
    names = [p[0] for p in sm.program(wi.RS, R, 1, 0, [(8 * j, 8 * j + 8) for j in range(R)], [(0, 8)], True)]
    assert names == (["notify", "direct_reduce_copy", "drain"] if R == 2 else
                     ["notify", "direct_reduce_send", "recv_reduce_send", "recv_reduce_copy", "drain"])
    colls = [wi.CollSpec(0, wi.RS, wi.F32, 20), wi.CollSpec(1, wi.RS, wi.BF16, 9), wi.CollSpec(2, wi.AR, wi.I32, 13)]
    for seed in range(4):
        g = np.random.default_rng(seed)
        orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]
        w = wi.Workload("direct_rs", R, colls, orders, seed=seed, cfg=95)
        S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=8, direct=True, lookahead=2, scan=bool(seed & 1)))
        posted = set()
        rng = np.random.default_rng(200 + seed)
        for _ in range(2_000_000):
            if S.done():
                break
            a = int(rng.integers(0, 3 * R))
            r = a % R
            if a < R:
                S.host_tick(r)
            elif a < 2 * R:
                S.daemons[r].mover_tick()
            else:
                S.daemons[r].tick()
            for d in S.daemons:
                for (c, seq) in d.cq:
                    if (d.r, c) not in posted:
                        posted.add((d.r, c))
                        f = S.fifo[c][d.r]
                        assert f.tail == f.head, "completion posted while the next rank still had something to read"
        assert S.done() and S.total_cqes() == R * len(colls)
        _check_data(S, w)


@pytest.mark.parametrize("direct", [False, True])
@pytest.mark.parametrize("R", [2, 3, 5])
def test_reduce_chain_in_the_model(R, direct):
    """The reduce collective as a chain root+1 -> ... -> root of one primitive per slice; with direct
    steps the first rank only notifies, the second reads the first one's send buffer, and a drain round
    holds every completion behind the neighbour's last read.  Only the root's recv buffer is written."""
    blocks = [(0, 8)] * R
    names = [sm.program(sm.RD, R, (2 + 1 + pos) % R, 2 % R, blocks, blocks, direct)[0][0] for pos in range(R)]
    if R == 2:
        assert names == (["notify", "direct_reduce_copy"] if direct else ["send", "recv_reduce_copy"])
    else:
        mid = ["recv_reduce_send"] * (R - 3)
        assert names == (["notify", "direct_reduce_send"] + mid + ["recv_reduce_copy"] if direct else
                         ["send", "recv_reduce_send"] + mid + ["recv_reduce_copy"])
    colls = [wi.CollSpec(0, wi.RD, wi.F32, 37, root=1 % R), wi.CollSpec(1, wi.RD, wi.BF16, 16, root=0),
             wi.CollSpec(2, wi.AR, wi.I32, 11), wi.CollSpec(3, wi.BC, wi.F16, 21, root=R - 1)]
    for seed in range(3):
        g = np.random.default_rng(seed)
        orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]
        w = wi.Workload("reduce_chain", R, colls, orders, seed=seed, cfg=96)
        S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=8, direct=direct, lookahead=2, scan=bool(seed & 1)))
        assert S.rounds[0] == 5 + (1 if direct else 0)
        posted = set()
        rng = np.random.default_rng(300 + seed)
        for _ in range(2_000_000):
            if S.done():
                break
            a = int(rng.integers(0, 3 * R))
            r = a % R
            if a < R:
                S.host_tick(r)
            elif a < 2 * R:
                S.daemons[r].mover_tick()
            else:
                S.daemons[r].tick()
            if direct:
                for d in S.daemons:
                    for (c, seq) in d.cq:
                        if (d.r, c) not in posted:
                            posted.add((d.r, c))
                            f = S.fifo[c][d.r]
                            assert f.tail == f.head, "completion posted while the next rank still had something to read"
        assert S.done() and S.total_cqes() == R * len(colls)
        _check_data(S, w)


def test_direct_broadcast_model_drains_after_the_last_slice():
    """The model's direct broadcast: one primitive per slice, one round more than slices, the drain;
    mixed with other kinds in random interleavings the values equal the data oracle's."""
    R = 4
    colls = [wi.CollSpec(0, wi.BC, wi.F32, 40, root=2), wi.CollSpec(1, wi.AR, wi.I32, 19), wi.CollSpec(2, wi.BC, wi.BF16, 7, root=0),
             wi.CollSpec(3, wi.AG, wi.F16, 6)]
    for seed in range(3):
        g = np.random.default_rng(seed)
        orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]
        w = wi.Workload("direct_bc", R, colls, orders, seed=seed, cfg=94)
        S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=8, direct=True, lookahead=2, scan=True))
        assert S.rounds[0] == 5 + 1 and S.rounds[2] == 1 + 1
        sm.run_random(S, seed + 7, max_ticks=3_000_000)
        assert S.total_cqes() == R * len(colls)
        _check_data(S, w)


# ---------------------------------------------------------------- priority-based ordering (Sec. 4.3)
_OPP, _SAME, _FOCUS = ((0, 1), (1, 0)), ((0, 1), (0, 1)), dict(lookahead=2, scan=True, focus=1)


@pytest.mark.parametrize("orders,var,prios", [(_OPP, dict(), (0, 1)), (_OPP, dict(scan=True, focus=1), (0, 1)),
                                              (_SAME, dict(scan=True, focus=1), (1, 0)), (_OPP, _FOCUS, (1, 0))])
def test_priority_ordering_exhaustive_interleavings_tiny(orders, var, prios):
    """Priority-based ordering (the SQ read before every pass, the queue kept sorted by the user's priority,
    priority first in a focused pass's ranking) keeps Alg. 1's liveness: over all interleavings of the
    circular-wait setting no reachable state is a deadlock and every one ends with the four CQEs, whichever
    of the two collectives is the more urgent one."""
    w = wi.config1(*orders, n=8)
    pol = sm.Policy(spin_init=2, spin_min=1, spin_max=2, boost=2, K=2, slice_elems=2 if var.get("scan") else 4,
                    priority_order=True, **var)
    S0 = _system(w, pol, data=False, priorities=prios)
    seen = sm.explore(S0, max_states=600_000)
    assert len(seen) > 20
    keys = list(seen)
    step = 1 if len(keys) < 1000 else 97
    for k in keys[::step]:
        T = seen[k].clone()
        assert not sm.is_deadlocked(T)
        sm.run_round_robin(T, max_ticks=50_000)
        assert T.total_cqes() == 4


@pytest.mark.parametrize("later_first", [True, False])
def test_priority_ordering_ranks_the_urgent_collective_first(later_first):
    """Four equal collectives queued in the order 0 .. 3 on both ranks, one queue per rank.  With later = more
    urgent the task queue is sorted 3, 2, 1, 0, every focused pass starts with the most urgent runnable one,
    and collective 3 completes first although it arrived last; with the priorities the other way round the
    order of completion is the order of arrival.  Values are the data oracle's either way."""
    n = 4
    colls = [wi.CollSpec(i, wi.AR, wi.I32, 48) for i in range(n)]
    w = wi.Workload("prio", 2, colls, [list(range(n))] * 2, seed=6, cfg=93)
    prios = list(range(n)) if later_first else [n - i for i in range(n)]
    S = _system(w, sm.Policy(spin_init=1, spin_min=1, spin_max=1, boost=1, K=2, slice_elems=4, scan=True, focus=1,
                             fetch_batch=0, priority_order=True), priorities=prios)
    S.submit_all()
    order = []
    for _ in range(5000):
        if S.done():
            break
        for d in S.daemons:
            was = d.in_pass
            d.tick()
            if d.in_pass and not was and d.ready:
                pr = [prios[d.taskq[i]] for i in d.ready]
                assert pr == sorted(pr, reverse=True)                       # most urgent runnable entry first
            assert [prios[c] for c in d.taskq] == sorted((prios[c] for c in d.taskq), reverse=True)   # sorted queue
            for c, _ in d.cq:
                if d.r == 0 and c not in order:
                    order.append(c)
    assert S.done() and S.total_cqes() == 2 * n
    assert order == (list(reversed(range(n))) if later_first else list(range(n))), order
    _check_data(S, w)


# ---------------------------------------------------------------- fold steps of an all-reduce
@pytest.mark.parametrize("var", [dict(), dict(scan=True), dict(lookahead=2, scan=True, focus=1), dict(fold_slice=2),
                                 dict(lookahead=2, scan=True, focus=1, fold_slice=2)])
@pytest.mark.parametrize("orders", [_OPP, _SAME])
def test_fold_steps_exhaustive_interleavings_tiny(orders, var):
    """All-reduces in fold steps (waits on all ranks through shared counters: published, folded) keep Alg. 1's liveness:
    in the circular-wait setting no reachable state -- over all interleavings of daemons, movers and host
    submissions -- is a deadlock, and every one of them ends with the four CQEs."""
    w = wi.config1(*orders, n=8)
    pol = sm.Policy(spin_init=2, spin_min=1, spin_max=2, boost=2, K=2, slice_elems=4, fold=True, **var)
    S0 = _system(w, pol, data=False)
    seen = sm.explore(S0, max_states=600_000)
    assert len(seen) > 20
    keys = list(seen)
    step = 1 if len(keys) < 1000 else 97
    for k in keys[::step]:
        T = seen[k].clone()
        assert not sm.is_deadlocked(T)
        sm.run_round_robin(T, max_ticks=50_000)
        assert T.total_cqes() == 4


def test_fold_steps_without_preemption_still_deadlock_on_opposite_orders():
    """The fold step waits for every rank to have fetched the collective: with one-entry task queues, opposite
    orders and no preemption each rank waits for the other to fetch what it will never fetch."""
    w = wi.config1((0, 1), (1, 0))
    S = _system(w, sm.Policy(preempt=False, K=2, slice_elems=256, taskq_cap=1, fold=True), data=False)
    with pytest.raises(TimeoutError):
        sm.run_round_robin(S, max_ticks=20_000)
    assert sm.is_deadlocked(S)


@pytest.mark.parametrize("var", [dict(), dict(lookahead=2, scan=True, focus=1, direct=True), dict(fold_slice=8),
                                 dict(lookahead=2, scan=True, focus=2, fold_slice=5)])
@pytest.mark.parametrize("seed", range(4))
def test_fold_steps_values_and_completion_order(var, seed):
    """All five kinds on three ranks in fold steps, random orders, random interleavings: the final
    buffers are the data oracle's -- the fold step's order of combination is the ring's -- and no rank posts a
    completion before every rank has finished the step with data (folded: the send buffers, which the others read, and
    the recv buffers, which the others write, are the caller's again after the completion)."""
    g = np.random.default_rng(seed)
    R = 3
    colls = [wi.CollSpec(0, wi.AR, wi.F32, 50), wi.CollSpec(1, wi.AG, wi.F16, 12), wi.CollSpec(2, wi.AR, wi.BF16, 33),
             wi.CollSpec(3, wi.BC, wi.BF16, 40, root=2), wi.CollSpec(4, wi.AR, wi.I32, 7), wi.CollSpec(5, wi.RS, wi.F32, 16),
             wi.CollSpec(6, wi.RD, wi.F16, 41, root=1)]
    orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]
    w = wi.Workload("fold", R, colls, orders, seed=seed, cfg=94)
    S = _system(w, sm.Policy(spin_init=2, spin_max=4, boost=2, K=2, slice_elems=8, fold=True, **var))
    ticks = 0
    while not S.done():
        a = int(g.integers(0, 3 * R))
        if a >= 2 * R:
            S.daemons[a - 2 * R].mover_tick()
        elif a >= R:
            S.host_tick(a - R)
        else:
            S.daemons[a].tick()
        for d in S.daemons:
            for c, _ in d.cq:                   # (every collective is invoked once here)
                k = colls[c].kind
                assert S.foldcnt[c][0] >= R
                if k in (wi.AR, wi.RS, wi.RD):
                    assert S.foldcnt[c][1] >= R * S.rounds[c]     # every rank has folded every slice: nobody reads a send buffer any more
                if k in (wi.AG, wi.BC):
                    assert S.foldcnt[c][2] >= R * S.rounds[c]     # every rank has gathered every slice
        ticks += 1
        assert ticks < 3_000_000
    assert S.total_cqes() == R * len(colls)
    _check_data(S, w)


@pytest.mark.parametrize("kinds", [(sm.RS, sm.AG), (sm.BC, sm.RD)])
def test_fold_steps_of_the_other_kinds_exhaustive_interleavings_tiny(kinds):
    """Two collectives of the other kinds in fold steps, issued in opposite orders on two ranks: no reachable state
    deadlocks and all end with the four CQEs."""
    colls = [wi.CollSpec(0, kinds[0], wi.F32, 8, root=1), wi.CollSpec(1, kinds[1], wi.F32, 8, root=0)]
    w = wi.Workload("fold2", 2, colls, [[0, 1], [1, 0]], seed=1, cfg=95)
    for var in (dict(), dict(lookahead=2, scan=True, focus=1), dict(lookahead=2, scan=True, focus=1, fold_slice=4)):
        S0 = _system(w, sm.Policy(spin_init=2, spin_min=1, spin_max=2, boost=2, K=2, slice_elems=4, fold=True, **var), data=False)
        seen = sm.explore(S0, max_states=600_000)
        assert len(seen) > 20
        keys = list(seen)
        for k in keys[::1 if len(keys) < 1000 else 97]:
            T = seen[k].clone()
            assert not sm.is_deadlocked(T)
            sm.run_round_robin(T, max_ticks=50_000)
            assert T.total_cqes() == 4


def test_fold_programs_move_fewer_blocks_than_the_ring():
    """Per rank, in chunks: the one data step of an all-reduce reads R and writes R (every input read once, every
    output written once); the second step only waits."""
    for R in (2, 3, 8):
        blocks = [(8 * j, 8 * j + 8) for j in range(R)]
        prog = sm.program(sm.AR, R, 1, 0, blocks, blocks, False, True)
        assert [n for n, _, _ in prog] == ["fold_scatter", "last_wait_red"]
        assert prog[0][1] == blocks[1] and prog[0][2] == blocks[1]        # rank r combines chunk r
