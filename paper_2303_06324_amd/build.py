"""Build the HIP library in-tree: hipcc -> paper_2303_06324_amd/libdfx.so (gfx950 only)."""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdfx.so")
SOURCES = ["dfx_daemon.hip", "dfx_host.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # never emit packed-fp32 instructions (hipcc flag; the host pass warns that it does not know it)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


ID_MARK = b"DFX_BUILD_ID="


def _id_inputs():
    root = os.path.dirname(HERE)
    files = sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".hip", ".h")))
    return files + [os.path.join(root, "include", "dfx.h")]


def source_id() -> str:
    """Hash of the sources the library is built from (csrc/*.hip, csrc/*.h, include/dfx.h) and of the
    compiler flags; baked into the library at build time (dfx_build_id) so that a library older than its
    sources is noticed instead of loaded."""
    import hashlib
    h = hashlib.sha256()
    for f in _id_inputs():
        h.update(os.path.basename(f).encode() + b"\0")
        with open(f, "rb") as fh:
            h.update(fh.read())
    h.update(" ".join(FLAGS + os.environ.get("DFX_EXTRA_DEFS", "").split()).encode())
    return h.hexdigest()[:16]


def built_id(path: str = LIB):
    """The id baked into a built library (read from the file, without loading it), or None."""
    try:
        with open(path, "rb") as fh:
            blob = fh.read()
    except OSError:
        return None
    at = blob.find(ID_MARK)
    if at < 0:
        return None
    return blob[at + len(ID_MARK):at + len(ID_MARK) + 16].decode("ascii", "replace")


def build(verbose: bool = False) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    extra = os.environ.get("DFX_EXTRA_DEFS", "").split()      # e.g. "-DDFX_UNROLL=4" for experiments
    extra = extra + ['-DDFX_BUILD_ID_STR="' + source_id() + '"']
    out = os.environ.get("DFX_BUILD_OUT", LIB)
    cmd = [hipcc] + FLAGS + extra + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", out + ".tmp", "-lpthread"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + err)
    os.replace(out + ".tmp", out)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return out


def build_c_client() -> str:
    """The plain C client of the boundary (tests/c_abi/c_client.c: gcc, no Python, no PyTorch) that the GPU
    tests run; links against the library built above."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "c_abi", "c_client.c")
    out = os.path.join(root, "tests", "c_abi", "c_client.bin")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(root, "include"),
           "-I" + os.path.join(rocm, "include"), src, "-o", out + ".tmp", "-L" + HERE, "-ldfx",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64",
           "-Wl,-rpath,$ORIGIN/../../paper_2303_06324_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + " ".join(cmd) + "\n" + res.stderr)
    os.replace(out + ".tmp", out)
    return out


def ensure_built() -> None:
    """Build what is missing or older than its sources, and nothing else (tests, smoke and the bench load
    what is there).  A library whose baked-in id differs from the sources' is rebuilt; where that is not
    possible (no compiler) the build raises, and so does loading the stale library (binding._load)."""
    if not os.path.exists(LIB) or built_id() != source_id():
        build()
    if not os.path.exists(os.path.join(os.path.dirname(HERE), "tests", "c_abi", "c_client.bin")):
        build_c_client()


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_c_client())
