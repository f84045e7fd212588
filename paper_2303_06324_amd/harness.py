"""Run a synthetic workload through the HIP library and fetch the results (GPU tests + bench).

Only marshalling lives here: buffers are torch byte tensors (PyTorch = device memory only),
every collective step runs in libdfx.so through the C ABI.
"""
from __future__ import annotations

import threading
import time
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import paper_2303_06324_amd as dfx
import workload_inputs as wi

SENTINEL = 0xA5
GUARD = 4096        # bytes of fill pattern in front of and behind every recv buffer


def make_config(**kw) -> "dfx.Config":
    cfg = dfx.config_default()
    for k, v in kw.items():
        if not hasattr(cfg, k):
            raise KeyError(k)
        setattr(cfg, k, v)
    return cfg


class DeviceWorkload:
    """Send/recv buffers of a Workload resident on the GPU.

    Every recv buffer lies between two guard zones of GUARD bytes that hold the fill pattern, so that a
    store outside the buffer (a tail that overruns, a slice that starts early) shows; check_untouched()
    looks at them and compares every send buffer with the bytes that were uploaded."""

    def __init__(self, w: wi.Workload, colls: Optional[Sequence[int]] = None, keep_host: bool = True,
                 sends: Optional[Dict[int, List[np.ndarray]]] = None):
        """sends: host send buffers per collective index (storage dtype), for inputs that the seeded recipe of
        workload_inputs does not draw (constructed values); default: wi.all_sends."""
        self.w = w
        self.idx = list(range(len(w.colls))) if colls is None else list(colls)
        self.send_host: Dict[int, List[np.ndarray]] = {}
        self.send: Dict[int, List[torch.Tensor]] = {}
        self.recv: Dict[int, List[torch.Tensor]] = {}       # the payload views (what the library is given)
        self._recv_alloc: Dict[int, List[torch.Tensor]] = {}  # guard | payload | guard
        self._recv_bytes: Dict[int, int] = {}
        for ci in self.idx:
            c = w.colls[ci]
            hs = sends[ci] if sends is not None else wi.all_sends(w, ci)
            assert len(hs) == w.R and all(h.size == c.send_elems(w.R) for h in hs)
            if keep_host:
                self.send_host[ci] = hs
            self.send[ci] = []
            for h in hs:
                b = h.view(np.uint8)
                t = torch.zeros(max(b.size, 16), dtype=torch.uint8, device="cuda")   # never a null pointer
                if b.size:
                    t[:b.size].copy_(torch.from_numpy(b))
                self.send[ci].append(t)
            nbytes = c.recv_elems(w.R) * wi.ELEM_BYTES[c.dtype]
            self._recv_bytes[ci] = nbytes
            self._recv_alloc[ci] = [torch.full((GUARD + max(nbytes, 16) + GUARD,), SENTINEL, dtype=torch.uint8, device="cuda")
                                    for _ in range(w.R)]
            self.recv[ci] = [t[GUARD:GUARD + max(nbytes, 16)] for t in self._recv_alloc[ci]]
        torch.cuda.synchronize()
        # the per-rank bursts of the workload's own issue orders, marshalled once (kept out of timed regions)
        self.bursts = None
        if colls is None:
            self.bursts = [dfx.Context.make_burst([w.colls[ci].coll_id for ci in w.orders[r]],
                                                  [self.send[ci][r].data_ptr() for ci in w.orders[r]],
                                                  [self.recv[ci][r].data_ptr() for ci in w.orders[r]],
                                                  w.delays_us[r] if w.delays_us else None)
                           for r in range(w.R)]

    def reset_recv(self):
        for ci in self.idx:
            for t in self._recv_alloc[ci]:
                t.fill_(SENTINEL)
        torch.cuda.synchronize()

    def results(self, ci: int) -> List[np.ndarray]:
        c = self.w.colls[ci]
        nbytes = self._recv_bytes[ci]
        return [t[:nbytes].cpu().numpy().view(wi.NP_STORAGE[c.dtype]) for t in self.recv[ci]]

    def check_untouched(self):
        """Nothing outside the recv buffers was written and no send buffer changed (the direct steps hand
        send buffers to the neighbour's movers, which must only read them)."""
        torch.cuda.synchronize()
        for ci in self.idx:
            nbytes = self._recv_bytes[ci]
            for r, t in enumerate(self._recv_alloc[ci]):
                if not bool((t[:GUARD] == SENTINEL).all()):
                    raise AssertionError(f"{self.w.name} coll {ci} rank {r}: bytes in front of the recv buffer were written")
                if not bool((t[GUARD + nbytes:] == SENTINEL).all()):
                    raise AssertionError(f"{self.w.name} coll {ci} rank {r}: bytes behind the recv buffer were written")
            if ci in self.send_host:
                for r, h in enumerate(self.send_host[ci]):
                    b = h.view(np.uint8)
                    if b.size and not torch.equal(self.send[ci][r][:b.size], torch.from_numpy(b).to("cuda")):
                        raise AssertionError(f"{self.w.name} coll {ci} rank {r}: the send buffer changed")


def prepare_all(ctx: "dfx.Context", w: wi.Workload, colls: Optional[Sequence[int]] = None, priorities=None):
    idx = range(len(w.colls)) if colls is None else colls
    for ci in idx:
        c = w.colls[ci]
        ctx.prepare(c.coll_id, c.kind, c.count, c.dtype, c.op, c.root,
                    0 if priorities is None else priorities[ci])


def _submit_retry(ctx, r, coll_id, s, d, deadline):
    while True:
        rc = ctx.submit(r, coll_id, s, d)
        if rc == dfx.OK:
            return
        if rc != dfx.ERR_SQ_FULL:
            raise dfx.DfxError(rc, f"dfx_submit(rank={r}, coll={coll_id})")
        ctx.poll(r, 0)          # lets the library restart a daemon that quit
        if time.monotonic() > deadline:
            raise TimeoutError("SQ stayed full")


def submit_round_robin(ctx: "dfx.Context", dw: DeviceWorkload, orders=None, timeout_s: float = 20.0):
    """One host thread walks the per-rank issue orders in lock step (rank 0's j-th, rank 1's j-th ...)."""
    w = dw.w
    orders = w.orders if orders is None else orders
    deadline = time.monotonic() + timeout_s
    n = max(len(o) for o in orders)
    for j in range(n):
        for r in range(w.R):
            if j < len(orders[r]):
                ci = orders[r][j]
                _submit_retry(ctx, r, w.colls[ci].coll_id, dw.send[ci][r].data_ptr(), dw.recv[ci][r].data_ptr(), deadline)


def submit_bursts(ctx: "dfx.Context", dw: DeviceWorkload, timeout_s: float = 30.0):
    """One host thread, one native burst per rank in turn (rank 0's whole issue order, then rank 1's ...): the
    workload's per-rank orders without a Python call per submission."""
    assert dw.bursts is not None
    for r in range(dw.w.R):
        burst = dw.bursts[r]
        if burst[4] is not None:
            burst = burst[:4] + (None,)
        n = ctx.submit_burst(r, burst, timeout_s)
        if n != burst[0]:
            raise dfx.DfxError(n if n < 0 else dfx.ERR_TIMEOUT, f"dfx_submit_many(rank={r}) -> {n}")


def submit_threads(ctx: "dfx.Context", dw: DeviceWorkload, orders=None, delays_us=None, timeout_s: float = 30.0,
                   barrier=None):
    """One host thread per rank, each with its own order and (optional) seeded delays.  Every thread makes one
    native call (pauses included), so the submitters really run concurrently; the bursts are marshalled before
    the threads start.  `barrier` (a threading.Barrier for R + 1 parties): every thread waits at it before its
    call, so that a caller who times the run can start its clock when all submitters are ready."""
    w = dw.w
    orders = w.orders if orders is None else orders
    errs = []
    bursts = []
    for r in range(w.R):
        if orders is w.orders and dw.bursts is not None and (delays_us is None or delays_us is w.delays_us):
            burst = dw.bursts[r]
            if delays_us is None and burst[4] is not None:
                burst = burst[:4] + (None,)
        else:
            burst = ctx.make_burst([w.colls[ci].coll_id for ci in orders[r]],
                                   [dw.send[ci][r].data_ptr() for ci in orders[r]],
                                   [dw.recv[ci][r].data_ptr() for ci in orders[r]],
                                   delays_us[r] if delays_us else None)
        bursts.append(burst)

    def work(r):
        try:
            if barrier is not None:
                barrier.wait()
            n = ctx.submit_burst(r, bursts[r], timeout_s)
            if n != bursts[r][0]:
                raise dfx.DfxError(n if n < 0 else dfx.ERR_TIMEOUT, f"dfx_submit_many_paced(rank={r}) -> {n}")
        except Exception as e:   # noqa: BLE001
            errs.append(e)

    ts = [threading.Thread(target=work, args=(r,)) for r in range(w.R)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    if errs:
        raise errs[0]


def run_workload(w: wi.Workload, cfg=None, mode: str = "roundrobin", timeout_s: float = 30.0,
                 dw: Optional[DeviceWorkload] = None, keep_ctx: bool = False):
    """Create a context, run every collective of w once in its per-rank orders, return
    (DeviceWorkload, per-rank stats, context or None)."""
    dw = dw or DeviceWorkload(w)
    ctx = dfx.Context(w.R, cfg)
    try:
        prepare_all(ctx, w)
        if mode == "threads":
            submit_threads(ctx, dw, delays_us=w.delays_us or None, timeout_s=timeout_s)
        else:
            submit_round_robin(ctx, dw, timeout_s=timeout_s)
        rc = ctx.wait_all(timeout_s)
        stop_rc = ctx.stop()
        stats = [ctx.stats(r) for r in range(w.R)]
        if rc != dfx.OK:
            raise dfx.DfxError(rc, f"dfx_wait_all (stop={stop_rc}, stats0={stats[0]})")
        dw.check_untouched()
    except Exception:
        try:                      # leave a trace of where every vrank stood
            ctx.stop()
            for r in range(w.R):
                st = ctx.stats(r)
                print(f"[harness] rank {r}: " + " ".join(f"{k}={v}" for k, v in st.items() if isinstance(v, int) and v))
        except Exception as e2:   # noqa: BLE001
            print("[harness] no stats:", e2)
        ctx.finalize()
        raise
    if keep_ctx:
        return dw, stats, ctx
    ctx.finalize()
    return dw, stats, None
