"""GPU parity on constructed values: the places where a reduction kernel can differ from the oracle
without random data ever showing it (subnormal inputs and results, exact cancellation to +0 / -0,
values within a binade of the largest finite one, constructed round-to-nearest-even ties, equal
values for maximum / minimum, int32 wraparound), for every dtype x reducing function x reducing
collective, bit for bit.  tests/test_crafted_inputs.py shows on the CPU that the inputs reach
those places."""
import numpy as np
import pytest

import workload_inputs as wi
from oracle import ring_data as rd
from tests import crafted_inputs as ci

pytestmark = pytest.mark.gpu


def _workload(R, seed, count_ar, count_rs):
    colls, sends = [], {}
    for kind in (wi.AR, wi.RS, wi.RD):
        for dtype in (wi.F32, wi.BF16, wi.F16, wi.I32):
            for op in (wi.SUM, wi.PROD, wi.MAX, wi.MIN):
                i = len(colls)
                count = count_rs if kind == wi.RS else count_ar
                c = wi.CollSpec(i, kind, dtype, count, root=(i * 5) % R, op=op)
                colls.append(c)
                sends[i] = ci.crafted_sends(dtype, op, R, c.send_elems(R), seed=seed + i)
    g = np.random.default_rng(seed)
    orders = [list(map(int, g.permutation(len(colls)))) for _ in range(R)]      # every rank its own order
    return wi.Workload(f"crafted_R{R}", R, colls, orders, seed=seed, cfg=77), sends


def _check_exact(dw, w):
    for i, c in enumerate(w.colls):
        want = rd.run_closed_form(c.kind, dw.send_host[i], c.dtype, c.root, c.op)
        got = dw.results(i)
        for r in range(w.R):
            if c.kind == wi.RD and r != c.root:
                assert np.all(got[r].view(np.uint8) == 0xA5), (i, r)
                continue
            if not np.array_equal(got[r].view(np.uint8), want[r].view(np.uint8)):
                eb = wi.ELEM_BYTES[c.dtype]
                u = {2: np.uint16, 4: np.uint32}[eb]
                bad = np.flatnonzero(got[r].view(u) != want[r].view(u))
                k = int(bad[0])
                ins = [hex(int(s.view(u)[k if c.kind != wi.RS else r * c.count + k])) for s in dw.send_host[i]]
                raise AssertionError(
                    f"{wi.KIND_NAMES[c.kind]} {wi.DTYPE_NAMES[c.dtype]} {wi.OP_NAMES[c.op]} R={w.R} rank {r}: {bad.size} "
                    f"elements differ, first at {k}: got {hex(int(got[r].view(u)[k]))} want {hex(int(want[r].view(u)[k]))} "
                    f"inputs {ins}")


@pytest.mark.parametrize("count_rs,knobs", [(15013, dict()), (15013, dict(fold_max_bytes=0)),
                                            (15016, dict(direct_min_bytes=0, fold_max_bytes=0, slot_bytes=4096, nslots=2, max_channels=4))],
                         ids=["defaults_fold_steps", "ring_through_slots", "ring_direct_steps_small_slots"])
@pytest.mark.parametrize("R", [8, 3])
def test_constructed_values_every_dtype_function_and_reducing_kind(R, count_rs, knobs):
    """48 collectives (all-reduce, reduce-scatter, reduce x four dtypes x four reducing functions) on
    constructed values, every rank submitting in its own order; ragged counts that span several
    channels, with the library defaults and with every kind on its direct steps, many slices per
    channel share and the fewest slots."""
    from paper_2303_06324_amd import harness as gh
    w, sends = _workload(R, 100 + R, count_ar=120011, count_rs=count_rs)   # (reduce-scatter blocks of 16-byte multiples take direct steps)
    dw = gh.DeviceWorkload(w, sends=sends)
    gh.run_workload(w, gh.make_config(**knobs), dw=dw, timeout_s=60.0)     # also checks guards and send buffers
    _check_exact(dw, w)
