"""Builds libhydragen.so (HIP, gfx950 only) in-tree with hipcc.  `python -m paper_2402_05099_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libhydragen.so")
SOURCES = ["api.hip", "prefix.hip", "prefix_wide.hip", "prefix_wide_d64.hip", "decode.hip", "merge.hip", "kvcache.hip", "decode_mfma.hip", "fused_small.hip", "ceilings.hip"]

# packed fp32 VALU forms are switched off for every device compile of this library
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option", "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


PER_SOURCE_FLAGS = {}   # source file name -> extra hipcc flags


def build(verbose: bool = True, extra_flags=(), out: str = LIB) -> str:
    """Compile every source to an object (sources may carry their own flags), then link the shared library.
    `out` other than the default names a variant build (e.g. one compiled with -DHG_TRACE, see prefix_wide.hip):
    select it at run time with HYDRAGEN_LIB=<path>."""
    objdir = os.path.join(PKG, "_build" if out == LIB else "_build_" + os.path.basename(out))
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()
    common = [f for f in HIPCC_FLAGS if f != "-shared"]
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        cmd = [cc, *common, *PER_SOURCE_FLAGS.get(src, []), *extra_flags, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
               "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd)))
        objs.append(obj)
    for cmd, pr in procs:
        if pr.wait() != 0:
            raise subprocess.CalledProcessError(pr.returncode, cmd)
    tmp = out + f".tmp{os.getpid()}"
    link = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.check_call(link)
    os.replace(tmp, out)
    return out


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [os.path.join(ROOT, "include", h) for h in ("hydragen.h", "hydragen_debug.h")]
    return any(os.path.getmtime(d) > t for d in deps)


if __name__ == "__main__":
    # usage: python -m paper_2402_05099_amd.build [--out variant.so] [extra hipcc flags...]
    argv = sys.argv[1:]
    target = LIB
    if "--out" in argv:
        i = argv.index("--out")
        target = os.path.abspath(argv[i + 1])
        del argv[i:i + 2]
    build(extra_flags=argv, out=target)
