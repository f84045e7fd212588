"""GPU tests of the scheduling behaviour: negative control, voluntary quit / restart, GPU
synchronisation between disordered collectives, priority ordering, SQ back-pressure, statistics."""
import time

import numpy as np
import pytest

import workload_inputs as wi
from oracle import ring_data as rd

pytestmark = pytest.mark.gpu


def _expect(dw, w, ci):
    c = w.colls[ci]
    want = rd.run_closed_form(c.kind, dw.send_host[ci], c.dtype, c.root, c.op)
    got = dw.results(ci)
    for r in range(w.R):
        assert np.array_equal(got[r].view(np.uint8), want[r].view(np.uint8)), (w.name, ci, r)


def test_negative_control_no_preemption_hits_watchdog():
    """Opposite issue orders with preemption disabled = the single-queue deadlock (Sec. 2.3, Fig. 1c;
    Sec. 6.1 reports 100 % for the non-preemptive library).  The in-kernel watchdog turns it into
    a timeout: every wave still leaves the kernel normally."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config1((0, 1), (1, 0))
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(2, gh.make_config(preempt=0, watchdog_ms=300, quit_idle_us=0, max_channels=2, chan_spread=0))
    try:
        gh.prepare_all(ctx, w)
        gh.submit_round_robin(ctx, dw)
        t0 = time.monotonic()
        assert ctx.wait_all(5.0) == dfx.ERR_TIMEOUT
        assert time.monotonic() - t0 < 4.0          # the watchdog, not the host deadline, ended it
        assert ctx.submit(0, 0, dw.send[0][0].data_ptr(), dw.recv[0][0].data_ptr()) == dfx.ERR_ABORTED
        st = [ctx.stats(r) for r in range(2)]
        assert sum(s["cqe_posted"] for s in st) == 0
    finally:
        assert ctx.finalize() == dfx.ERR_ABORTED


def test_same_order_without_preemption_completes():
    from paper_2303_06324_amd import harness as gh
    w = wi.config1((0, 1), (0, 1))
    dw, stats, _ = gh.run_workload(w, gh.make_config(preempt=0, watchdog_ms=2000, max_channels=2, chan_spread=0))
    for ci in range(2):
        _expect(dw, w, ci)
    assert sum(s["preemptions"] for s in stats) == 0


@pytest.mark.parametrize("direct_min_bytes", [2 << 20, 0])
def test_voluntary_quit_and_event_driven_restart(direct_min_bytes):
    """Sec. 4.4: the daemon leaves when idle and is started again by the next SQE; contexts survive."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.Workload("quit", 8, [wi.CollSpec(0, wi.AR, wi.F32, 200000)], [[0]] * 8, seed=5, cfg=70)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config(quit_idle_us=300, direct_min_bytes=direct_min_bytes))
    try:
        gh.prepare_all(ctx, w)
        launches = []
        for it in range(3):
            dw.reset_recv()
            gh.submit_round_robin(ctx, dw)
            assert ctx.wait_all(10.0) == dfx.OK
            _expect(dw, w, 0)
            time.sleep(0.05)                       # far longer than the quit period
            ms, done = ctx.last_launch_ms()
            launches.append(done)
        assert launches[0] >= 1 and launches[2] >= launches[0] + 2
        st = ctx.stats(0)
        assert st["quits"] > 0
    finally:
        assert ctx.finalize() == dfx.OK


def test_device_synchronize_between_disordered_collectives():
    """Sec. 2.3 'GPU synchronization related' deadlock (Fig. 1d) / Sec. 6.1 second program: a
    device-wide synchronisation between collectives issued in opposite orders.  The stuck daemon
    quits voluntarily, the synchronisation returns, the remaining SQEs restart the daemon."""
    import torch
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config1((0, 1), (1, 0), n=50000)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(2, gh.make_config(quit_idle_us=500, max_channels=4))
    try:
        gh.prepare_all(ctx, w)
        assert ctx.submit(0, 0, dw.send[0][0].data_ptr(), dw.recv[0][0].data_ptr()) == dfx.OK   # rank 0: A
        assert ctx.submit(1, 1, dw.send[1][1].data_ptr(), dw.recv[1][1].data_ptr()) == dfx.OK   # rank 1: B
        t0 = time.monotonic()
        torch.cuda.synchronize()                   # returns only once the daemon has left the GPU
        assert time.monotonic() - t0 < 5.0
        assert ctx.submit(0, 1, dw.send[1][0].data_ptr(), dw.recv[1][0].data_ptr()) == dfx.OK   # rank 0: B
        assert ctx.submit(1, 0, dw.send[0][1].data_ptr(), dw.recv[0][1].data_ptr()) == dfx.OK   # rank 1: A
        assert ctx.wait_all(10.0) == dfx.OK
        for ci in range(2):
            _expect(dw, w, ci)
        assert ctx.stats(0)["quits"] > 0
    finally:
        ctx.finalize()


@pytest.mark.parametrize("path", ["ring", "fold"])
@pytest.mark.parametrize("single_queue", [0, 1])
def test_eight_allreduces_in_a_new_random_order_every_iteration(path, single_queue):
    """The shape of the first deadlock program of Sec. 6.1: eight vranks, eight all-reduces of 256 B .. 1 MiB, two
    hundred iterations, in every iteration every vrank submits the eight in a fresh random order of its own (a
    non-preemptive library deadlocks on the first disagreement; Sec. 6.1 reports 100 %).  All iterations complete,
    the values are the oracle's, and the daemon got there by preempting (with one shared queue per vrank, the
    single-queue setting of Sec. 2.3, and with the collectives spread over the workgroups)."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    R, iters = 8, 200
    sizes = [256, 1024, 4096, 16384, 65536, 262144, 524288, 1 << 20]
    colls = [wi.CollSpec(i, wi.AR, wi.F32, nb // 4) for i, nb in enumerate(sizes)]
    w = wi.Workload("deadlock_program_1", R, colls, [list(range(8))] * R, seed=61, cfg=53)
    dw = gh.DeviceWorkload(w)
    knobs = dict(fold_max_bytes=0) if path == "ring" else {}
    if single_queue:
        knobs.update(chan_spread=0, max_channels=1)
    ctx = dfx.Context(R, gh.make_config(**knobs))      # (default idle quit: reading results back waits for the daemon to leave)
    g = np.random.default_rng(2024)
    try:
        gh.prepare_all(ctx, w)
        for it in range(iters):
            orders = [list(map(int, g.permutation(8))) for _ in range(R)]
            gh.submit_round_robin(ctx, dw, orders=orders, timeout_s=30)
            assert ctx.wait_all(30.0) == dfx.OK, it
            if it in (0, iters - 1):
                for ci in range(8):
                    _expect(dw, w, ci)
                if it == 0:       # wipe the results (on the current stream only: the daemon's stream never drains)
                    import torch
                    for ci in range(8):
                        for r in range(R):
                            dw.recv[ci][r].zero_()
                    torch.cuda.current_stream().synchronize()
        assert ctx.stop() == dfx.OK
        st = [ctx.stats(r) for r in range(R)]
        assert sum(s["cqe_posted"] for s in st) == iters * 8 * R
        assert sum(s["preemptions"] for s in st) > iters          # it did have to switch away from stuck collectives
    finally:
        assert ctx.finalize() == dfx.OK


def test_priority_ordering_policy():
    """Sec. 4.3 priority-based ordering: later-arriving collectives get higher priority (the DP
    overlap scheme); everything still completes and matches."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config3(n_buckets=12, bucket_bytes=1 << 20, seed=8)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config(order_policy=1))
    try:
        gh.prepare_all(ctx, w, priorities=list(range(12)))
        gh.submit_round_robin(ctx, dw)
        assert ctx.wait_all(30.0) == dfx.OK
        for ci in range(12):
            _expect(dw, w, ci)
    finally:
        ctx.finalize()


def _completion_order(order_policy, priorities, n_colls=8, nbytes=8 << 20, late_last_ms=0.0, **knobs):
    """n equal all-reduces on ONE channel per vrank (one task queue per rank), submitted 0, 1, ... on every rank;
    returns the order in which vrank 0's completions are seen by a tight poll loop.  The daemon's launch waits
    behind a kernel that only sleeps, so every submission is in the SQs when the daemon first looks (host
    scheduling has no say); with late_last_ms the last collective is submitted that much later, while the
    others are under way."""
    import time
    import torch
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    R = 8
    colls = [wi.CollSpec(i, wi.AR, wi.F32, nbytes // 4) for i in range(n_colls)]
    w = wi.Workload("prio_order", R, colls, [list(range(n_colls))] * R, seed=31, cfg=50)
    dw = gh.DeviceWorkload(w)
    stream = torch.cuda.Stream()                     # default priority
    ctx = dfx.Context(R, gh.make_config(order_policy=order_policy, max_channels=1, chan_spread=0, quit_idle_us=0, **knobs),
                      stream=stream.cuda_stream)
    order = []
    try:
        gh.prepare_all(ctx, w, priorities=priorities)
        slept = torch.cuda.Event()
        with torch.cuda.stream(stream):
            torch.cuda._sleep(20_000_000)            # some milliseconds: the submissions below take microseconds
            slept.record(stream)
        first = n_colls - 1 if late_last_ms else n_colls
        gh.submit_round_robin(ctx, dw, orders=[list(range(first))] * R, timeout_s=30)
        if late_last_ms:
            deadline = time.monotonic() + 10.0
            while not slept.query():                 # the sleeping kernel has ended: the daemon starts on the others now
                assert time.monotonic() < deadline
            time.sleep(late_last_ms * 1e-3)
            gh.submit_round_robin(ctx, dw, orders=[[n_colls - 1]] * R, timeout_s=30)
        deadline = time.monotonic() + 30.0
        while len(order) < n_colls:
            order += [cid for cid, _ in ctx.poll(0, 64)]
            assert time.monotonic() < deadline
        assert ctx.wait_all(30.0) == dfx.OK
        assert ctx.stop() == dfx.OK
        for ci in range(n_colls):
            _expect(dw, w, ci)
    finally:
        ctx.finalize()
    return order


def _out_of_order_pairs(order, want):
    """Pairs of completions that came in the opposite order to `want` (a list of all ids); 0 = exactly `want`."""
    rank = {c: i for i, c in enumerate(want)}
    return sum(1 for i in range(len(order)) for j in range(i + 1, len(order)) if rank[order[i]] > rank[order[j]])


@pytest.mark.parametrize("path", ["ring", "fold"])
def test_priority_ordering_decides_who_completes_first(path):
    """Eight equal all-reduces (8 MiB, one channel: about a millisecond each) queued on every vrank in the order
    0 .. 7.  Under FIFO ordering the one submitted first completes first and the one submitted last does
    not; under priority ordering with later = more urgent (the DP-overlap scheme of Sec. 4.3) the one
    submitted last completes first; with the priorities the other way round the order is the FIFO one again.
    As rings every collective's opening step is runnable from the start, so the order is exact.  In fold steps a
    collective is runnable once ALL vranks have fetched it, and the eight per-collective counters of the first burst
    fill in any order: a daemon that looks in between starts on what is runnable then, so one completion may come out
    of turn (at most 7 of the 28 pairs swapped; a policy that is ignored swaps all 28, chance 14)."""
    knobs = dict(fold_max_bytes=0) if path == "ring" else {}
    up, down = list(range(8)), list(range(7, -1, -1))

    def check(order, want):
        if path == "ring":
            assert order[:4] == want[:4] and order.index(want[-1]) > 3, (order, want)
        else:
            assert order.index(want[0]) <= 1 and order.index(want[-1]) >= 6 and _out_of_order_pairs(order, want) <= 7, (order, want)

    check(_completion_order(0, None, **knobs), up)
    check(_completion_order(1, list(range(8)), **knobs), down)
    check(_completion_order(1, [8 - i for i in range(8)], **knobs), up)
    # the same with Alg. 1's own queue handling (no readiness scan: the sorted queue and the thresholds decide)
    alg1 = _completion_order(1, list(range(8)), scan_min=0, **knobs)
    assert alg1.index(7) < alg1.index(0), alg1


def test_priority_ordering_lets_a_late_urgent_collective_overtake():
    """Seven all-reduces (milliseconds each) are under way when an eighth, more urgent one is submitted 0.3 ms later: under
    priority ordering it overtakes those queued and begun before it; under FIFO ordering it is among the last two to complete."""
    # (rings: cut into 256 KiB slices, so that the urgent one gets the movers slice by slice; in fold steps a step of a
    # collective on ONE channel is a single job of megabytes, and what is posted is not taken back)
    fifo = _completion_order(0, None, late_last_ms=0.3, fold_max_bytes=0)
    assert fifo.index(7) >= 6, fifo       # (it may finish neck and neck with the one queued just before it)
    prio = _completion_order(1, list(range(8)), late_last_ms=0.3, fold_max_bytes=0)
    assert prio.index(7) <= 1, prio


def test_sq_backpressure_and_poll_interface():
    """A 4-entry SQ with 40 collectives: submit returns SQ_FULL until every workgroup of the rank
    has read a slot (Sec. 5); dfx_poll hands out each completion exactly once."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config5(n_colls=40, seed=9, R=4)
    dw = gh.DeviceWorkload(w)
    import torch
    stream = torch.cuda.Stream()                     # default priority
    ctx = dfx.Context(4, gh.make_config(sq_depth=4, max_channels=8), stream=stream.cuda_stream)
    try:
        gh.prepare_all(ctx, w)
        # The daemon's launch queues behind a kernel that just waits for a while, so nothing reads the
        # SQ yet: four entries of vrank 0 fit, the fifth finds the ring full.
        with torch.cuda.stream(stream):
            torch.cuda._sleep(20_000_000)
        for j in range(4):
            ci = w.orders[0][j]
            assert ctx.submit(0, ci, dw.send[ci][0].data_ptr(), dw.recv[ci][0].data_ptr()) == dfx.OK
        ci = w.orders[0][4]
        assert ctx.submit(0, ci, dw.send[ci][0].data_ptr(), dw.recv[ci][0].data_ptr()) == dfx.ERR_SQ_FULL
        full = 1
        seen = [set() for _ in range(4)]
        pos = [4, 0, 0, 0]
        deadline = time.monotonic() + 30
        while any(p < 40 for p in pos) or any(len(s) < 40 for s in seen):
            for r in range(4):
                if pos[r] < 40:
                    ci = w.orders[r][pos[r]]
                    rc = ctx.submit(r, ci, dw.send[ci][r].data_ptr(), dw.recv[ci][r].data_ptr())
                    if rc == dfx.OK:
                        pos[r] += 1
                    else:
                        assert rc == dfx.ERR_SQ_FULL
                        full += 1
                for cid, seq in ctx.poll(r, 8):
                    assert cid not in seen[r] and seq == 0
                    seen[r].add(cid)
            assert time.monotonic() < deadline
        assert full > 0
        for ci in range(40):
            _expect(dw, w, ci)
        assert ctx.poll(0, 8) == []
    finally:
        ctx.finalize()


def test_stats_are_consistent():
    from paper_2303_06324_amd import harness as gh
    w = wi.config3(n_buckets=6, bucket_bytes=512 << 10, seed=12)
    dw, stats, _ = gh.run_workload(w, gh.make_config(spin_init=8, spin_min=1, spin_max=32, spin_boost=2, trace=1,
                                                      chan_spread=0, scan_min=0))   # shared queues, polled in turn
    for s in stats:
        assert s["cqe_posted"] == 6
        # every preemption either saves the dynamic context or skips the save because nothing had moved
        # (a save without a preemption happens only when the grid is aborted, which this run is not)
        assert s["preemptions"] == s["ctx_saves"] + s["lazy_skips"]
        assert s["ctx_loads"] + s["ctx_slot_hits"] >= s["preemptions"]
        assert s["max_taskq"] <= 6
    assert sum(s["preemptions"] for s in stats) > 0 and sum(s["lazy_skips"] for s in stats) > 0
    assert sum(s["switch_samples"] for s in stats) > 0
    assert all(0.0 < s["switch_us_p50"] < 100.0 for s in stats if s["switch_samples"])


@pytest.mark.parametrize("placement", [0, 1])
def test_sq_placements(placement):
    """SQ in pinned host memory (the paper's placement, Sec. 5) and in fine-grained device memory
    written by the host through the PCIe BAR: same results; the device placement needs a large BAR."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config4(n_colls=12, min_bytes=4096, max_bytes=1 << 20, seed=21)
    try:
        dw, stats, _ = gh.run_workload(w, gh.make_config(sq_in_device=placement), mode="threads", timeout_s=30.0)
    except dfx.DfxError as e:
        if placement == 1 and e.status == dfx.ERR_NO_RESOURCES:
            pytest.skip("device does not report a large BAR")
        raise
    for ci in range(12):
        _expect(dw, w, ci)


@pytest.mark.parametrize("direct_min_bytes", [2 << 20, 0])
def test_stop_with_outstanding_work_and_resume(direct_min_bytes):
    """dfx_stop (exit SQE, Sec. 4.4) while collectives are stuck: their contexts survive in the
    context buffer (Sec. 4.5) and the next start resumes them (also with the direct gather steps,
    whose published recv-buffer addresses must survive in the connectors)."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config3(n_buckets=4, bucket_bytes=1 << 20, seed=15)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config(quit_idle_us=0, direct_min_bytes=direct_min_bytes))
    try:
        gh.prepare_all(ctx, w)
        for ci in range(4):                      # only ranks 0..5 submit: nothing can complete
            for r in range(6):
                assert ctx.submit(r, ci, dw.send[ci][r].data_ptr(), dw.recv[ci][r].data_ptr()) == dfx.OK
        time.sleep(0.02)
        assert ctx.stop() == dfx.OK
        assert ctx.poll(0, 8) == []
        for cycle in range(2):                   # an empty start/stop cycle in between
            assert ctx.start() == dfx.OK
            assert ctx.stop() == dfx.OK
        for ci in range(4):
            for r in (6, 7):
                assert ctx.submit(r, ci, dw.send[ci][r].data_ptr(), dw.recv[ci][r].data_ptr()) == dfx.OK
        assert ctx.wait_all(20.0) == dfx.OK
        for ci in range(4):
            _expect(dw, w, ci)
    finally:
        assert ctx.finalize() == dfx.OK


def test_focused_passes_keep_a_workgroup_longer_on_one_collective():
    """focus_bytes (the default path's stand-in for Sec. 4.3's stickiness): with sixteen disordered buckets as rings,
    a scanned pass that visits the furthest-along collective first and ends after its byte budget makes a workgroup
    stay longer with one collective than passes that visit every runnable collective once in queue order.  Measured
    on the per-workgroup timeline (trace = 3): mean length of the runs of consecutive primitives of one collective,
    2.8-3.0 with the default budget against 2.4-2.5 without (the effect is real and small; the values are the
    oracle's either way)."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config3(n_buckets=16, bucket_bytes=4 << 20)
    dw = gh.DeviceWorkload(w)
    run_len = {}
    for focus in (128 << 10, 0):
        ctx = dfx.Context(8, gh.make_config(quit_idle_us=0, trace=3, fold_max_bytes=0, focus_bytes=focus))
        try:
            gh.prepare_all(ctx, w)
            gh.submit_bursts(ctx, dw, timeout_s=60)
            assert ctx.wait_all(60.0) == dfx.OK
            assert ctx.stop() == dfx.OK
            for ci in (0, 7, 15):
                _expect(dw, w, ci)
            runs = []
            for wg in range(0, 8 * gh.make_config().max_channels, 5):
                samples, _ = ctx.trace_read(wg)
                ids = [(s >> 48) & 0xfff for s in samples if (s >> 60) != 15]
                if len(ids) >= 16:
                    runs.append(len(ids) / (1 + sum(1 for a, b in zip(ids, ids[1:]) if a != b)))
            assert len(runs) >= 20
            run_len[focus] = float(np.mean(runs))
        finally:
            assert ctx.finalize() == dfx.OK
    assert run_len[128 << 10] > 1.08 * run_len[0], run_len


def test_primitive_timeline_trace():
    """trace = 3: one sample per executed primitive and per wait that ended in preemption; every
    workgroup that served the collective reports its 2R-1 primitives per slice, in sequence order,
    with data phases that do not overlap in time."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.Workload("timeline", 8, [wi.CollSpec(0, wi.AR, wi.F32, 1 << 20)], [[0]] * 8, seed=21, cfg=71)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config(trace=3, quit_idle_us=0))
    try:
        gh.prepare_all(ctx, w)
        gh.submit_round_robin(ctx, dw)
        assert ctx.wait_all(20.0) == dfx.OK
        assert ctx.stop() == dfx.OK
        _expect(dw, w, 0)
        info = ctx.coll_info(0)
        cmax = gh.make_config().max_channels
        served = 0
        for wg in range(8 * cmax):
            samples, tick_us = ctx.trace_read(wg)
            assert 0.0 < tick_us < 1.0
            prims = [s for s in samples if (s >> 60) != 15]
            if not prims:
                continue
            served += 1
            nprim = info["nprim"] - 1          # the all-reduce's last step (drain) moves nothing and leaves no sample
            assert len(prims) == info["rounds"] * nprim
            # slices are taken in windows of two: primitive p of both slices, then p + 1, ...
            order = []
            for base in range(0, info["rounds"], 2):
                width = min(2, info["rounds"] - base)
                order += [p for p in range(nprim) for _ in range(width)]
            assert [s >> 60 for s in prims] == order
            assert all(((s >> 48) & 0xfff) == 0 for s in samples)
            end = None
            for s in prims:
                start, dur = s & 0xffffffff, (s >> 32) & 0xffff
                assert end is None or ((start - end) & 0xffffffff) < (1 << 31)
                end = (start + dur) & 0xffffffff
        assert served == 8 * info["nchan"]
    finally:
        assert ctx.finalize() == dfx.OK


@pytest.mark.parametrize("cq_mode", [0, 1, 2])
def test_cq_variants_deliver_every_completion_once(cq_mode):
    """The three completion queues of Sec. 5 (CAS slot array, vanilla ring, 64-bit packed ring) behind a
    16-slot CQ that must wrap many times: 200 collectives per rank, every CQE handed out exactly once."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.config5(n_colls=200, seed=23)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config(cq_mode=cq_mode, cq_slots=16))
    try:
        gh.prepare_all(ctx, w)
        seen = [dict() for _ in range(8)]
        pos = [0] * 8
        deadline = time.monotonic() + 60
        while any(p < 200 for p in pos) or any(len(s) < 200 for s in seen):
            for r in range(8):
                for _ in range(4):
                    if pos[r] < 200:
                        ci = w.orders[r][pos[r]]
                        rc = ctx.submit(r, ci, dw.send[ci][r].data_ptr(), dw.recv[ci][r].data_ptr())
                        if rc == dfx.OK:
                            pos[r] += 1
                        else:
                            assert rc == dfx.ERR_SQ_FULL
                for cid, seq in ctx.poll(r, 64):
                    assert cid not in seen[r] and seq == 0
                    seen[r][cid] = seq
            assert time.monotonic() < deadline
        for ci in range(200):
            _expect(dw, w, ci)
        st = ctx.stats(0)
        assert st["cqe_posted"] == 200 and st["cqe_us"] > 0.0
    finally:
        assert ctx.finalize() == dfx.OK


def test_callback_poller_thread():
    """Sec. 3.1: a poller thread reads the CQEs and runs the callback; nothing is left for dfx_poll, and
    the thread restarts a daemon that quit while work was outstanding."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    import threading
    w = wi.config3(n_buckets=8, bucket_bytes=256 << 10, seed=24)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config(quit_idle_us=200))
    got, lock, all_done = [], threading.Lock(), threading.Event()

    def on_done(rank, coll_id, seq):
        with lock:
            got.append((rank, coll_id, seq))
            if len(got) == 2 * 8 * 8:
                all_done.set()

    try:
        gh.prepare_all(ctx, w)
        ctx.set_callback(on_done)
        for rep in range(2):
            for ci in range(8):                      # ranks 0..6 first: the daemon gets stuck and quits
                for r in range(7):
                    assert ctx.submit(r, ci, dw.send[ci][r].data_ptr(), dw.recv[ci][r].data_ptr()) == dfx.OK
            time.sleep(0.01)
            for ci in range(8):
                assert ctx.submit(7, ci, dw.send[ci][7].data_ptr(), dw.recv[ci][7].data_ptr()) == dfx.OK
            assert ctx.wait_all(20.0) == dfx.OK
        assert all_done.wait(10.0)
        for r in range(8):
            assert ctx.poll(r, 8) == []
        with lock:
            assert sorted(got) == sorted((r, ci, rep) for rep in range(2) for r in range(8) for ci in range(8))
        ctx.set_callback(None)
        for ci in range(8):
            _expect(dw, w, ci)
    finally:
        assert ctx.finalize() == dfx.OK


def test_submit_all_is_one_invocation_on_every_vrank():
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.Workload("submit_all", 8, [wi.CollSpec(0, wi.AR, wi.I32, 70001)], [[0]] * 8, seed=31, cfg=72)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(8, gh.make_config())
    try:
        gh.prepare_all(ctx, w)
        ptrs = ctx.make_all([t.data_ptr() for t in dw.send[0]], [t.data_ptr() for t in dw.recv[0]])
        for it in range(3):
            assert ctx.submit_all(0, ptrs) == dfx.OK
            if it == 0:
                assert ctx.submit_all(0, ptrs) == dfx.ERR_BUSY        # the invocation is outstanding on vrank 0
            assert ctx.wait_all(20.0) == dfx.OK
            _expect(dw, w, 0)
        assert ctx.stop() == dfx.OK                      # counters are written back when the workgroups leave
        assert [s["cqe_posted"] for s in (ctx.stats(r) for r in range(8))] == [3] * 8
    finally:
        assert ctx.finalize() == dfx.OK


def test_paced_burst_honours_its_delays():
    """dfx_submit_many_paced waits delays_ns[i] before entry i (the issue-time jitter of the
    disordered-invocation experiments, Sec. 6.1); data must still equal the oracle's."""
    import threading
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    R, n = 4, 6
    colls = [wi.CollSpec(i, wi.AR, wi.I32, 3000 + 17 * i) for i in range(n)]
    w = wi.Workload("paced", R, colls, [list(range(n))] * R, seed=77, cfg=73)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(R, gh.make_config())
    try:
        gh.prepare_all(ctx, w)
        delay_us = 20000.0
        bursts = []
        for r in range(R):
            order = list(range(n)) if r % 2 == 0 else list(reversed(range(n)))
            bursts.append(ctx.make_burst(order, [dw.send[ci][r].data_ptr() for ci in order],
                                         [dw.recv[ci][r].data_ptr() for ci in order],
                                         [delay_us if r == 0 else 0.0] * n))
        out = [None] * R
        took = [0.0] * R

        def work(r):
            t0 = time.monotonic()
            out[r] = ctx.submit_burst(r, bursts[r])
            took[r] = time.monotonic() - t0

        th = [threading.Thread(target=work, args=(r,)) for r in range(R)]
        for t in th:
            t.start()
        for t in th:
            t.join()
        assert out == [n] * R
        assert took[0] >= n * delay_us * 1e-6            # every pause was taken
        assert max(took[1:]) < n * delay_us * 1e-6       # and only where one was asked for
        assert ctx.wait_all(20.0) == dfx.OK
        for ci in range(n):
            _expect(dw, w, ci)
    finally:
        assert ctx.finalize() == dfx.OK


def test_host_error_paths_leave_the_context_usable():
    """Argument errors are reported by the host side before anything reaches the SQ; a context that
    has reported them still runs a collective correctly afterwards."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    w = wi.Workload("errs", 4, [wi.CollSpec(0, wi.AR, wi.F32, 5001), wi.CollSpec(1, wi.BC, wi.I32, 333, root=2)],
                    [[0, 1]] * 4, seed=9, cfg=74)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(4, gh.make_config(max_colls=8))
    try:
        s, d = dw.send[0][0].data_ptr(), dw.recv[0][0].data_ptr()
        assert ctx.submit(0, 0, s, d) == dfx.ERR_NOT_PREPARED
        gh.prepare_all(ctx, w)
        for bad in [dict(coll_id=8), dict(coll_id=-1), dict(kind=5), dict(dtype=4), dict(op=4),
                    dict(kind=dfx.BROADCAST, root=4), dict(kind=dfx.REDUCE, root=-1),
                    dict(priority=40000), dict(count=(1 << 40) + 1), dict(coll_id=0)]:
            a = dict(coll_id=2, kind=dfx.ALLREDUCE, count=64, dtype=dfx.F32, op=dfx.SUM, root=0, priority=0)
            a.update(bad)
            with pytest.raises(dfx.DfxError) as ei:
                ctx.prepare(**a)
            assert ei.value.status == dfx.ERR_INVALID_ARG, bad
        assert ctx.submit(4, 0, s, d) == dfx.ERR_INVALID_ARG
        assert ctx.submit(-1, 0, s, d) == dfx.ERR_INVALID_ARG
        assert ctx.submit(0, 8, s, d) == dfx.ERR_INVALID_ARG
        assert ctx.submit(0, 2, s, d) == dfx.ERR_NOT_PREPARED
        assert ctx.submit(0, 0, 0, d) == dfx.ERR_INVALID_ARG
        assert ctx.submit(0, 0, s, 0) == dfx.ERR_INVALID_ARG
        assert ctx.submit(0, 0, s + 4, d) == dfx.ERR_INVALID_ARG          # user buffers are 16-byte aligned
        assert ctx.submit(0, 0, s, d + 8) == dfx.ERR_INVALID_ARG
        assert ctx.wait(0, 9) == dfx.ERR_INVALID_ARG
        assert ctx.wait(7, 0) == dfx.ERR_INVALID_ARG
        with pytest.raises(dfx.DfxError):
            ctx.poll(5)
        with pytest.raises(dfx.DfxError):
            ctx.coll_info(2)
        st = [ctx.stats(r) for r in range(4)]
        assert sum(x["launches"] + x["sqe_fetched"] for x in st) == 0       # nothing reached a queue
        gh.submit_round_robin(ctx, dw)
        assert ctx.wait_all(20.0) == dfx.OK
        for ci in range(2):
            _expect(dw, w, ci)
    finally:
        assert ctx.finalize() == dfx.OK


def test_two_contexts_take_turns_on_the_device():
    """Two daemon grids cannot be resident together (each fills the device and spins on its own
    flags), so a context's daemon is started only when no other context's is in flight: both
    contexts finish their collectives, and a daemon that never quits makes the other one wait
    until it is stopped."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    wa = wi.Workload("turn_a", 8, [wi.CollSpec(0, wi.AR, wi.I32, 150001)], [[0]] * 8, seed=41, cfg=75)
    wb = wi.Workload("turn_b", 4, [wi.CollSpec(0, wi.AG, wi.F16, 4099)], [[0]] * 4, seed=42, cfg=76)
    da, db = gh.DeviceWorkload(wa), gh.DeviceWorkload(wb)
    A = dfx.Context(8, gh.make_config(quit_idle_us=300))
    B = dfx.Context(4, gh.make_config(quit_idle_us=300))
    try:
        gh.prepare_all(A, wa)
        gh.prepare_all(B, wb)
        pa = A.make_all([t.data_ptr() for t in da.send[0]], [t.data_ptr() for t in da.recv[0]])
        pb = B.make_all([t.data_ptr() for t in db.send[0]], [t.data_ptr() for t in db.recv[0]])
        for it in range(3):
            assert A.submit_all(0, pa) == dfx.OK
            assert B.submit_all(0, pb) == dfx.OK       # B's daemon is put off while A's is in flight
            assert B.wait_all(20.0) == dfx.OK          # ... and started from here once A's has quit
            assert A.wait_all(20.0) == dfx.OK
            _expect(da, wa, 0)
            _expect(db, wb, 0)
        assert A.stop() == dfx.OK and B.stop() == dfx.OK
        assert A.stats(0)["launches"] >= 1 and B.stats(0)["launches"] >= 1
    finally:
        ra, rb = A.finalize(), B.finalize()
    assert (ra, rb) == (dfx.OK, dfx.OK)
    # a daemon that never quits keeps the device until it is stopped
    A = dfx.Context(8, gh.make_config(quit_idle_us=0))
    B = dfx.Context(4, gh.make_config(quit_idle_us=300))
    try:
        gh.prepare_all(A, wa)
        gh.prepare_all(B, wb)
        pa = A.make_all([t.data_ptr() for t in da.send[0]], [t.data_ptr() for t in da.recv[0]])
        pb = B.make_all([t.data_ptr() for t in db.send[0]], [t.data_ptr() for t in db.recv[0]])
        assert A.submit_all(0, pa) == dfx.OK and A.wait_all(20.0) == dfx.OK
        assert B.submit_all(0, pb) == dfx.OK
        assert B.wait_all(0.2) == dfx.ERR_TIMEOUT
        assert B.stats(0)["launches"] == 0
        assert A.stop() == dfx.OK
        assert B.wait_all(20.0) == dfx.OK
        _expect(db, wb, 0)
    finally:
        ra, rb = A.finalize(), B.finalize()
    assert (ra, rb) == (dfx.OK, dfx.OK)


def test_submit_all_is_all_or_nothing_and_bursts_keep_their_order():
    """dfx_submit_all takes every vrank's entry or none: with one vrank's invocation of the collective still
    outstanding it returns BUSY and leaves the other vranks free to be submitted one by one.  A burst
    (dfx_submit_many) with the same id twice stops at the repeat and reports how many went in."""
    from paper_2303_06324_amd import harness as gh
    import paper_2303_06324_amd as dfx
    R = 8
    w = wi.Workload("all_or_nothing", R, [wi.CollSpec(0, wi.AR, wi.I32, 5000), wi.CollSpec(1, wi.AR, wi.F32, 777)], [[0, 1]] * R, seed=5, cfg=52)
    dw = gh.DeviceWorkload(w)
    ctx = dfx.Context(R, gh.make_config())
    try:
        gh.prepare_all(ctx, w)
        ptrs = ctx.make_all([dw.send[0][r].data_ptr() for r in range(R)], [dw.recv[0][r].data_ptr() for r in range(R)])
        assert ctx.submit(3, 0, dw.send[0][3].data_ptr(), dw.recv[0][3].data_ptr()) == dfx.OK
        assert ctx.submit_all(0, ptrs) == dfx.ERR_BUSY            # vrank 3 has it outstanding: nobody is submitted
        for r in range(R):
            if r != 3:
                assert ctx.submit(r, 0, dw.send[0][r].data_ptr(), dw.recv[0][r].data_ptr()) == dfx.OK
        assert ctx.wait_all(20.0) == dfx.OK
        _expect(dw, w, 0)
        # a burst of vrank 0: ids 1, 0, 1 -- the third is a repeat of an outstanding one
        burst = ctx.make_burst([1, 0, 1], [dw.send[1][0].data_ptr(), dw.send[0][0].data_ptr(), dw.send[1][0].data_ptr()],
                               [dw.recv[1][0].data_ptr(), dw.recv[0][0].data_ptr(), dw.recv[1][0].data_ptr()])
        assert ctx.submit_burst(0, burst, 5.0) == 2
        for r in range(1, R):
            assert ctx.submit(r, 1, dw.send[1][r].data_ptr(), dw.recv[1][r].data_ptr()) == dfx.OK
            assert ctx.submit(r, 0, dw.send[0][r].data_ptr(), dw.recv[0][r].data_ptr()) == dfx.OK
        assert ctx.wait_all(20.0) == dfx.OK
        _expect(dw, w, 0)
        _expect(dw, w, 1)
    finally:
        assert ctx.finalize() == dfx.OK


def test_plain_c_client_of_the_boundary():
    """A C program (gcc, no Python, no PyTorch, hipMalloc'ed buffers) drives the library through include/dfx.h
    alone: the circular wait of two all-reduces, then an all-reduce, a direct reduce-scatter and a broadcast
    on eight vranks in per-rank orders (rings and chains), then a small all-reduce in fold steps two hundred times
    inside a resident daemon; all checked against element-wise integer sums written out in C."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "c_client.bin")
    assert os.path.exists(exe), "the C client is not built (python -m paper_2303_06324_amd.build)"
    res = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    assert res.returncode == 0, (res.returncode, res.stdout, res.stderr)
    assert "circular wait ok" in res.stdout and "eight ranks ok" in res.stdout and "small all-reduce ok" in res.stdout
    print(res.stdout)
