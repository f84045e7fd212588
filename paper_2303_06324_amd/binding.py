"""Thin ctypes binding of the dfx C ABI (include/dfx.h): argument marshalling only.

Every step of the hot path runs in the HIP library; nothing here computes, and there is no
fallback: importing this module without the built library raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdfx.so")

ALLREDUCE, ALLGATHER, REDUCESCATTER, BROADCAST, REDUCE = 0, 1, 2, 3, 4
F32, BF16, F16, I32 = 0, 1, 2, 3
SUM, PROD, MAX, MIN = 0, 1, 2, 3

OK = 0
ERR_INVALID_ARG, ERR_NOT_PREPARED, ERR_BUSY, ERR_SQ_FULL = -1, -2, -3, -4
ERR_TIMEOUT, ERR_HIP, ERR_NO_RESOURCES, ERR_ABORTED, ERR_TOO_LARGE = -5, -6, -7, -8, -9
NOALLOC_MAX_BYTES = 1 << 30


class Config(C.Structure):
    _fields_ = [(n, C.c_uint32) for n in (
        "struct_bytes", "max_channels", "max_colls", "sq_depth", "cq_slots", "nslots", "slot_bytes",
        "chan_min_bytes", "spin_init", "spin_min", "spin_max", "spin_boost", "preempt", "watchdog_ms",
        "quit_idle_us", "sq_in_device", "wg_map", "order_policy", "trace", "fetch_batch")] + [("pool_bytes", C.c_uint64), ("scan_min", C.c_uint32), ("chan_spread", C.c_uint32), ("cq_mode", C.c_uint32), ("sq_eager", C.c_uint32), ("window", C.c_uint32), ("focus_bytes", C.c_uint32), ("direct", C.c_uint32), ("direct_min_bytes", C.c_uint32), ("fold_max_bytes", C.c_uint32), ("fold_slice_bytes", C.c_uint32), ("reserved0", C.c_uint32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "preemptions", "ctx_loads", "ctx_slot_hits", "ctx_saves", "lazy_skips", "polls", "prims", "sqe_fetched",
        "cqe_posted", "max_taskq", "passes", "quits", "launches", "switch_samples")] + [(n, C.c_double) for n in (
        "switch_us_p50", "switch_us_p99", "switch_us_mean", "save_us_mean", "load_us_mean", "wait_us", "data_us",
        "publish_us")] + [("scan_skips", C.c_uint64), ("cqe_us", C.c_double), ("advance_us_mean", C.c_double),
                          ("setup_us_mean", C.c_double), ("clock_read_us", C.c_double), ("sqe_us", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


CALLBACK = C.CFUNCTYPE(None, C.c_void_p, C.c_int, C.c_uint32, C.c_uint32)


class Cqe(C.Structure):
    _fields_ = [("coll_id", C.c_uint32), ("seq", C.c_uint32)]


class DfxError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {strerror(status)} ({status})")


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it first (python -m paper_2303_06324_amd.build); "
                          "there is no CPU fallback")
    # PyTorch (device memory and streams) ships its own HIP runtime: load it first so that this
    # library binds to the same runtime instance instead of a second copy.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    from . import build as _build
    have, want = _build.built_id(LIB_PATH), _build.source_id()
    if have != want and os.environ.get("DFX_ANY_BUILD") != "1":      # (the switch is for A/B runs of experiment builds)
        raise ImportError(f"{LIB_PATH} was built from other sources (id {have}, sources {want}): rebuild it "
                          "(python -m paper_2303_06324_amd.build)")
    lib = C.CDLL(LIB_PATH)
    vp, i, u64, sz = C.c_void_p, C.c_int, C.c_uint64, C.c_size_t
    sig = {
        "dfx_config_default": ([C.POINTER(Config)], i),
        "dfx_init": ([C.POINTER(vp), i, C.POINTER(Config), vp], i),
        "dfx_prepare": ([vp, i, i, sz, i, i, i, i], i),
        "dfx_submit": ([vp, i, i, vp, vp], i),
        "dfx_submit_many": ([vp, i, i, C.POINTER(C.c_int), C.POINTER(vp), C.POINTER(vp), u64], i),
        "dfx_submit_all": ([vp, i, C.POINTER(vp), C.POINTER(vp), u64], i),
        "dfx_submit_many_paced": ([vp, i, i, C.POINTER(C.c_int), C.POINTER(vp), C.POINTER(vp), C.POINTER(u64), u64], i),
        "dfx_poll": ([vp, i, C.POINTER(Cqe), i], i),
        "dfx_wait": ([vp, i, i, u64], i),
        "dfx_wait_all": ([vp, u64], i),
        "dfx_start": ([vp], i),
        "dfx_stop": ([vp], i),
        "dfx_stats": ([vp, i, C.POINTER(Stats)], i),
        "dfx_coll_info": ([vp, i] + [C.POINTER(C.c_uint32)] * 4, i),
        "dfx_last_launch_ms": ([vp, C.POINTER(C.c_float), C.POINTER(u64)], i),
        "dfx_trace_read": ([vp, C.c_uint32, C.POINTER(u64), C.c_uint32, C.POINTER(C.c_double)], i),
        "dfx_set_callback": ([vp, CALLBACK, vp], i),
        "dfx_finalize": ([vp], i),
        "dfx_last_hip_error": ([vp], i),
        "dfx_last_init_error": ([], i),
        "dfx_strerror": ([i], C.c_char_p),
        "dfx_build_id": ([], C.c_char_p),
        "dfx_copy_calibrate": ([vp, vp, sz, vp, C.POINTER(C.c_float)], i),
        "dfx_check_geometry": ([i, C.POINTER(Config), i, sz, i, i, i, i, C.c_uint32, C.c_char_p, sz], i),
        "dfx_collective_noalloc": ([i, i, sz, i, i, i, C.POINTER(vp), C.POINTER(vp), vp, vp], i),
    }
    for name, (args, res) in sig.items():
        f = getattr(lib, name)
        f.argtypes, f.restype = args, res
    return lib


_lib = _load()


def build_id() -> str:
    return _lib.dfx_build_id().decode()


def strerror(status: int) -> str:
    return _lib.dfx_strerror(status).decode()


def config_default() -> Config:
    cfg = Config()
    _lib.dfx_config_default(C.byref(cfg))
    return cfg


class Context:
    """One dfx context = R virtual ranks on the current GPU. Methods mirror the C entry points."""

    def __init__(self, nranks: int, cfg: Optional[Config] = None, stream: Optional[int] = None):
        self._h = C.c_void_p()
        self.nranks = nranks
        rc = _lib.dfx_init(C.byref(self._h), nranks, C.byref(cfg) if cfg is not None else None,
                           C.c_void_p(stream) if stream else None)
        if rc != OK:
            self._h = C.c_void_p()
            raise DfxError(rc, f"dfx_init (hipError {_lib.dfx_last_init_error()})")

    def prepare(self, coll_id: int, kind: int, count: int, dtype: int, op: int = SUM, root: int = 0,
                priority: int = 0) -> None:
        rc = _lib.dfx_prepare(self._h, coll_id, kind, count, dtype, op, root, priority)
        if rc != OK:
            raise DfxError(rc, "dfx_prepare")

    def submit(self, rank: int, coll_id: int, sendbuf: int, recvbuf: int) -> int:
        """Returns the status (OK, ERR_SQ_FULL, ERR_BUSY ...) without raising: callers retry."""
        return _lib.dfx_submit(self._h, rank, coll_id, C.c_void_p(sendbuf), C.c_void_p(recvbuf))

    def make_all(self, sendbufs, recvbufs):
        """Marshal the per-vrank pointers of one invocation once."""
        return (C.c_void_p * self.nranks)(*sendbufs), (C.c_void_p * self.nranks)(*recvbufs)

    def submit_all(self, coll_id: int, ptrs, timeout_s: float = 30.0) -> int:
        """One invocation on every vrank in one call; ptrs from make_all. Returns the status."""
        return _lib.dfx_submit_all(self._h, coll_id, ptrs[0], ptrs[1], int(timeout_s * 1e9))

    @staticmethod
    def make_burst(coll_ids, sendbufs, recvbufs, delays_us=None):
        """Marshal a burst once (C arrays), so that submitting it costs no Python work; delays_us[i] is a
        pause before entry i."""
        n = len(coll_ids)
        d = (C.c_uint64 * n)(*[int(x * 1000.0) for x in delays_us]) if delays_us is not None else None
        return n, (C.c_int * n)(*coll_ids), (C.c_void_p * n)(*sendbufs), (C.c_void_p * n)(*recvbufs), d

    def submit_burst(self, rank: int, burst, timeout_s: float = 30.0) -> int:
        """Burst submission in C (the GIL is released for the whole call). Returns the count submitted."""
        n, ids, sb, rb, d = burst
        return _lib.dfx_submit_many_paced(self._h, rank, n, ids, sb, rb, d, int(timeout_s * 1e9))

    def submit_many(self, rank: int, coll_ids, sendbufs, recvbufs, timeout_s: float = 30.0) -> int:
        return self.submit_burst(rank, self.make_burst(coll_ids, sendbufs, recvbufs), timeout_s)

    def poll(self, rank: int, max_n: int = 64) -> List[Tuple[int, int]]:
        buf = (Cqe * max_n)()
        n = _lib.dfx_poll(self._h, rank, buf, max_n)
        if n < 0:
            raise DfxError(n, "dfx_poll")
        return [(buf[k].coll_id, buf[k].seq) for k in range(n)]

    def wait(self, rank: int, coll_id: int, timeout_s: float = 10.0) -> int:
        return _lib.dfx_wait(self._h, rank, coll_id, int(timeout_s * 1e9))

    def wait_all(self, timeout_s: float = 10.0) -> int:
        return _lib.dfx_wait_all(self._h, int(timeout_s * 1e9))

    def start(self) -> int:
        return _lib.dfx_start(self._h)

    def stop(self) -> int:
        return _lib.dfx_stop(self._h)

    def stats(self, rank: int) -> dict:
        s = Stats()
        rc = _lib.dfx_stats(self._h, rank, C.byref(s))
        if rc != OK:
            raise DfxError(rc, "dfx_stats")
        return s.as_dict()

    def coll_info(self, coll_id: int) -> dict:
        v = [C.c_uint32() for _ in range(4)]
        rc = _lib.dfx_coll_info(self._h, coll_id, *[C.byref(x) for x in v])
        if rc != OK:
            raise DfxError(rc, "dfx_coll_info")
        return dict(nchan=v[0].value, slot_bytes=v[1].value, rounds=v[2].value, nprim=v[3].value)

    def last_launch_ms(self) -> Tuple[float, int]:
        ms, n = C.c_float(), C.c_uint64()
        rc = _lib.dfx_last_launch_ms(self._h, C.byref(ms), C.byref(n))
        if rc != OK:
            raise DfxError(rc, "dfx_last_launch_ms")
        return ms.value, n.value

    def set_callback(self, fn) -> None:
        """fn(rank, coll_id, seq) is called on the library's poller thread for every completion; None stops it."""
        if fn is None:
            rc = _lib.dfx_set_callback(self._h, C.cast(None, CALLBACK), None)
            self._cb = None
        else:
            cb = CALLBACK(lambda user, rank, coll_id, seq: fn(rank, coll_id, seq))
            rc = _lib.dfx_set_callback(self._h, cb, None)
            self._cb = cb           # keep the trampoline alive while the thread may call it
        if rc != OK:
            raise DfxError(rc, "dfx_set_callback")

    def trace_read(self, wg: int, max_samples: int = 4096) -> Tuple[list, float]:
        buf = (C.c_uint64 * max_samples)()
        tick = C.c_double()
        n = _lib.dfx_trace_read(self._h, wg, buf, max_samples, C.byref(tick))
        if n < 0:
            raise DfxError(n, "dfx_trace_read")
        return list(buf[:n]), tick.value

    def last_hip_error(self) -> int:
        return _lib.dfx_last_hip_error(self._h)

    def finalize(self) -> int:
        if not self._h:
            return OK
        rc = _lib.dfx_finalize(self._h)
        self._h = C.c_void_p()
        return rc

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.finalize()
        return False

    def __del__(self):
        try:
            self.finalize()
        except Exception:
            pass


def copy_calibrate(src: int, dst: int, nbytes: int, stream: Optional[int] = None) -> float:
    """Plain copy kernel of known traffic; returns its duration in milliseconds (HIP events)."""
    ms = C.c_float()
    rc = _lib.dfx_copy_calibrate(C.c_void_p(src), C.c_void_p(dst), nbytes, C.c_void_p(stream) if stream else None,
                                 C.byref(ms))
    if rc != OK:
        raise DfxError(rc, "dfx_copy_calibrate")
    return ms.value


def collective_noalloc(nranks: int, kind: int, count: int, dtype: int, op: int, root: int, sendbufs, recvbufs,
                       status_dev: int = 0, stream: Optional[int] = None) -> int:
    """One collective on every vrank through the entry point that allocates nothing; only enqueues work on
    `stream`.  Returns the status (OK, ERR_TOO_LARGE, ERR_BUSY ...) without raising."""
    sb = (C.c_void_p * nranks)(*sendbufs)
    rb = (C.c_void_p * nranks)(*recvbufs)
    return _lib.dfx_collective_noalloc(nranks, kind, count, dtype, op, root, sb, rb,
                                       C.c_void_p(status_dev) if status_dev else None,
                                       C.c_void_p(stream) if stream else None)


def check_geometry(nranks: int, kind: int, count: int, dtype: int, op: int = SUM, root: int = 0, coll_id: int = 0,
                   wg_map: int = 0, cfg: Optional[Config] = None) -> str:
    """Host-side self-check of the kernel's index arithmetic (no GPU needed); returns "" or the first violation."""
    buf = C.create_string_buffer(512)
    rc = _lib.dfx_check_geometry(nranks, C.byref(cfg) if cfg is not None else None, kind, count, dtype, op, root,
                                 coll_id, wg_map, buf, 512)
    return "" if rc == OK else (buf.value.decode() or strerror(rc))
