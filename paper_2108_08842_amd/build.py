"""Builds libeden_hip.so in-tree with hipcc for gfx950.  `python -m paper_2108_08842_amd.build`."""
import glob
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
LIB = os.path.join(PKG, "libeden_hip.so")
OBJ_DIR = os.path.join(ROOT, "_build")
SOURCES = ["eden_tables.cpp", "eden_kernels.hip", "eden_kernels_wg.hip", "eden_kernels_lo14.hip", "eden_api.hip"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (proc.stdout + proc.stderr).splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    return out


def _stale(src: str, obj: str) -> bool:
    if not os.path.exists(obj):
        return True
    csrc = os.path.join(PKG, "csrc")
    deps = [src, os.path.join(ROOT, "include", "eden.h")] + [os.path.join(csrc, f) for f in os.listdir(csrc) if f.endswith(".h")]
    return any(os.path.getmtime(dep) > os.path.getmtime(obj) for dep in deps)


def wide_stores_with_scalar_offset(obj_dir: str = OBJ_DIR):
    """Lines of the device assembly the last build left in `obj_dir` that store more than 64 bits through a buffer
    descriptor with the offset in a scalar register.  The compiler assumes that the data registers of such a store may be
    overwritten by the next instruction; on the MI355X that stored the next instruction's result instead of the data, in
    some lanes, when the memory pipeline was busy.  The kernels keep the whole offset in the vector register (the compiler
    then inserts the wait states); this check fails the build if one slips back in."""
    bad = []
    for path in sorted(glob.glob(os.path.join(obj_dir, "*-hip-amdgcn-amd-amdhsa-gfx950.s"))):
        for n, line in enumerate(open(path), 1):
            m = re.match(r"\s*buffer_store_dwordx[34]\s+v\[\d+:\d+\],\s*\S+,\s*s\[\d+:\d+\],\s*(\S+)", line)
            if m and m.group(1).rstrip(",") != "0":
                bad.append(f"{os.path.basename(path)}:{n}: {line.strip()}")
    return bad


def build(verbose: bool = True, incremental: bool = False) -> str:
    """Compiles every source to an object file (in parallel, one hipcc each) and links the shared library.
    `incremental`: skip sources whose object file is newer than the source and every header."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    common = [hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
              # packed fp32 instructions are kept off on the test machines
              "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
              "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(PKG, "csrc")]
    objs = [os.path.join(OBJ_DIR, s + ".o") for s in SOURCES]
    # the .hip sources also leave their device assembly beside the objects (checked below)
    cmds = [common + (["-save-temps=obj"] if s.endswith(".hip") else []) + ["-c", os.path.join(PKG, "csrc", s), "-o", o]
            for s, o in zip(SOURCES, objs) if not incremental or _stale(os.path.join(PKG, "csrc", s), o)]
    with ThreadPoolExecutor(max(1, len(cmds))) as pool:
        outs = list(pool.map(lambda c: _run(c, verbose), cmds))
    bad = wide_stores_with_scalar_offset()
    if bad:
        raise RuntimeError("128-bit buffer stores with a scalar offset register (see wide_stores_with_scalar_offset):\n" + "\n".join(bad))
    outs.append(_run([hipcc_path(), "--offload-arch=gfx950", "-fPIC", "-shared"] + objs + ["-o", LIB], verbose))
    if verbose:
        text = "\n".join(o for o in outs if o.strip())
        if text:
            print(text)
    return LIB


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv)
    sys.exit(0)
