"""CPU checks of the boundary: the C-ABI library loads and exports every symbol that include/dfx.h
declares, argument validation works without a GPU, and the product package never imports the oracle."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dfx.h")
LIB = os.path.join(ROOT, "paper_2303_06324_amd", "libdfx.so")


def _declared():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dfx_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_boundary_calls():
    names = _declared()
    for need in ("dfx_init", "dfx_prepare", "dfx_submit", "dfx_poll", "dfx_wait", "dfx_finalize", "dfx_stats",
                 "dfx_strerror"):
        assert need in names


def test_library_exports_every_declared_symbol():
    assert os.path.exists(LIB), "build first: python -m paper_2303_06324_amd.build"
    lib = ctypes.CDLL(LIB)
    for name in _declared():
        assert hasattr(lib, name), f"{name} declared in dfx.h but not exported"


def test_config_struct_matches_header_size():
    import paper_2303_06324_amd as dfx
    cfg = dfx.config_default()
    assert cfg.struct_bytes == ctypes.sizeof(dfx.Config) == 136
    assert cfg.nslots >= 2 and cfg.max_colls <= 4096 and cfg.preempt == 1
    assert dfx.strerror(0) == "ok" and "timeout" in dfx.strerror(dfx.ERR_TIMEOUT)


def test_argument_validation_without_gpu():
    import paper_2303_06324_amd as dfx
    lib = dfx.binding._lib
    h = ctypes.c_void_p()
    assert lib.dfx_init(None, 8, None, None) == dfx.ERR_INVALID_ARG
    assert lib.dfx_init(ctypes.byref(h), 0, None, None) == dfx.ERR_INVALID_ARG
    assert lib.dfx_init(ctypes.byref(h), 65, None, None) == dfx.ERR_INVALID_ARG
    bad = dfx.config_default()
    bad.nslots = 1          # a one-slot connector cannot run a fused recv+send ring
    assert lib.dfx_init(ctypes.byref(h), 8, ctypes.byref(bad), None) == dfx.ERR_INVALID_ARG
    for k in (0, 1, 3, 128):    # not a power of two in 2 .. 64 (0 once sent the window clamp into an endless loop)
        bad = dfx.config_default()
        bad.nslots = k
        assert lib.dfx_init(ctypes.byref(h), 8, ctypes.byref(bad), None) == dfx.ERR_INVALID_ARG
    bad = dfx.config_default()
    bad.fold_slice_bytes = 100      # not a multiple of 16 bytes
    assert lib.dfx_init(ctypes.byref(h), 8, ctypes.byref(bad), None) == dfx.ERR_INVALID_ARG
    bad = dfx.config_default()
    bad.sq_depth = 100
    assert lib.dfx_init(ctypes.byref(h), 8, ctypes.byref(bad), None) == dfx.ERR_INVALID_ARG
    bad = dfx.config_default()
    bad.struct_bytes = 4
    assert lib.dfx_init(ctypes.byref(h), 8, ctypes.byref(bad), None) == dfx.ERR_INVALID_ARG
    assert lib.dfx_submit(None, 0, 0, None, None) == dfx.ERR_INVALID_ARG
    assert lib.dfx_finalize(None) == dfx.ERR_INVALID_ARG


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2303_06324_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt, f"{f} mentions the oracle"


def test_c_client_is_built_against_the_library():
    """The plain C client of the boundary (built by build(), run by a GPU test) exists and resolves the
    library through its run path."""
    import subprocess
    exe = os.path.join(ROOT, "tests", "c_abi", "c_client.bin")
    assert os.path.exists(exe), "run python -m paper_2303_06324_amd.build first"
    out = subprocess.run(["ldd", exe], capture_output=True, text=True, timeout=60).stdout
    line = [l for l in out.splitlines() if "libdfx.so" in l]
    assert line and "paper_2303_06324_amd/libdfx.so" in line[0] and "not found" not in line[0], out


def test_build_module_runs_without_the_library():
    """Importing the package or its build module does not load the binding (which needs the built library), so
    the build can run in a tree that has no library yet; any use of the binding loads it, and fails loudly
    when the library is missing."""
    import subprocess
    import sys
    code = ("import sys, paper_2303_06324_amd, paper_2303_06324_amd.build; "
            "assert 'paper_2303_06324_amd.binding' not in sys.modules; "
            "paper_2303_06324_amd.ALLREDUCE; assert 'paper_2303_06324_amd.binding' in sys.modules")
    res = subprocess.run([sys.executable, "-c", code], cwd=ROOT, capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stderr
    src = open(os.path.join(ROOT, "paper_2303_06324_amd", "binding.py")).read()
    assert "raise ImportError" in src and "no CPU fallback" in src


def test_library_carries_the_id_of_its_sources():
    """The loaded library was built from the sources in the tree (a stale one is refused at load)."""
    import paper_2303_06324_amd as dfx
    from paper_2303_06324_amd import build as b
    assert dfx.build_id() == b.source_id() == b.built_id()
    assert len(dfx.build_id()) == 16
