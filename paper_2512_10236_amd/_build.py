"""Builds libficco.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libficco.so")
SOURCES = ["ficco_gemm.hip", "ficco_reduce.hip", "ficco_plan.hip", "ficco_engines.hip", "ficco_api.hip", "ficco_static.hip"]
HEADERS = ["ficco_internal.h", "ficco_plan.h", os.path.join("..", "..", "include", "ficco.h")]

# packed fp32 instructions are switched off for all device code (they have misbehaved on the test machines)
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function",
         "-Wno-inline-asm"]     # the direct-to-LDS loader names M0 as clobbered; the back end remarks that M0 is reserved


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(os.path.join(CSRC, f)) > t for f in SOURCES + HEADERS)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source and link the shared library. Returns its path."""
    if not force and not is_stale():
        return LIB
    return _compile(LIB, CSRC, [], verbose)


def build_variant(out: str, defines: list[str], verbose: bool = False) -> str:
    """A measuring build with extra -D switches (the timing-only ablations FICCO_ABL_* and the in-kernel clock
    probes FICCO_PROBE of ficco_gemm.hip), linked to `out`; load it with FICCO_LIBRARY=<out>. The in-tree
    library is not touched. Example:
        python -c "from paper_2512_10236_amd import _build; _build.build_variant('/tmp/libficco_nobar.so', ['FICCO_ABL_NOBAR'])"
    """
    import tempfile
    with tempfile.TemporaryDirectory() as objdir:
        return _compile(os.path.abspath(out), objdir, ["-D" + d for d in defines], verbose)


def _compile(lib: str, objdir: str, extra: list[str], verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "not a recognized feature" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    tmp = lib + f".tmp{os.getpid()}"
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs + ["-lhsa-runtime64"]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed: " + r.stdout)
    os.replace(tmp, lib)
    return lib


if __name__ == "__main__":
    print(build(verbose=True))
