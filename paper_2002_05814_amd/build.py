"""Builds libhop.so (the C-ABI reduce library) for gfx950 with hipcc, in-tree.

The reduce kernels are instantiated once per (element type, op) pair from
csrc/hop_kernels_inst.hip; the translation units are compiled side by side and
linked into one shared library.
"""
from __future__ import annotations

import hashlib
import os
import shutil
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhop.so")

# -packed-fp32-ops is switched off for the device pass (the host pass does not know the
# feature and says so: harmless).
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-fast-math", "-ffp-contract=off",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def _units():
    """(source, extra flags, object name) of every translation unit."""
    units = [("hop_api.hip", [], "hop_api.o"), ("hop_kernels.hip", [], "hop_kernels.o")]
    for dt in range(3):
        for op in range(3):
            units.append(("hop_kernels_inst.hip", ["-DHOP_INST_DT=%d" % dt, "-DHOP_INST_OP=%d" % op],
                          "hop_inst_%d_%d.o" % (dt, op)))
    return units


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)


def _sources_digest(src: str, extra) -> str:
    """Hash of a translation unit's inputs: its source, every header beside it, the public header, the flags."""
    h = hashlib.sha256()
    names = [os.path.join(CSRC, src)] + sorted(
        os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith((".h", ".hpp")))
    names.append(os.path.join(os.path.dirname(HERE), "include", "hop.h"))
    for name in names:
        with open(name, "rb") as f:
            h.update(f.read())
    h.update(" ".join([*HIPCC_FLAGS, *extra]).encode())
    return h.hexdigest()[:20]


def build(verbose: bool = False, jobs: int | None = None, object_cache: str | None = None) -> str:
    """Compile every HIP source into paper_2002_05814_amd/libhop.so.

    Without object_cache everything is compiled afresh. With it (a directory), objects whose inputs are
    unchanged since an earlier build are taken from there: for edit-compile loops during development.
    """
    jobs = jobs or max(1, min(8, os.cpu_count() or 1))
    cc = hipcc()
    with tempfile.TemporaryDirectory(prefix="hop_build_") as tmpdir:
        objs = []
        cmds = []
        for src, extra, obj in _units():
            if object_cache:
                os.makedirs(object_cache, exist_ok=True)
                out = os.path.join(object_cache, "%s.%s.o" % (obj[:-2], _sources_digest(src, extra)))
                objs.append(out)
                if os.path.exists(out):
                    continue
            else:
                out = os.path.join(tmpdir, obj)
                objs.append(out)
            cmds.append([cc, *HIPCC_FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", out])
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        tmp = LIB + ".tmp.%d" % os.getpid()
        _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp], verbose)
        os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    import sys
    cache = os.path.join(os.path.dirname(HERE), "_build") if "--incremental" in sys.argv[1:] else None
    print(build(verbose="--quiet" not in sys.argv[1:], object_cache=cache))
