"""Builds libsentencekv.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libsentencekv.so")
# profiling build (-DSKV_PHASE_STAMPS): the decode kernels record the wall clock at marked places, see csrc/skv_stamps.h;
# built by `python -m paper_2504_00970_amd._build --stamps`, loaded by `bench.py --phase-stamps`
LIB_STAMPS = os.path.join(HERE, "libsentencekv_stamps.so")
SOURCES = ["api.hip", "prefill.hip", "decode.hip", "retain.hip"]
HEADERS = [os.path.join(CSRC, "skv_internal.h"), os.path.join(CSRC, "skv_device.h"), os.path.join(CSRC, "skv_stamps.h"),
           os.path.join(INCLUDE, "sentencekv.h")]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions stay off: the compiler would otherwise form them from scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def stale(lib: str = "") -> bool:
    lib = lib or LIB
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, stamps: bool = False) -> str:
    """Compile the library: one hipcc process per source file, side by side, then one link.  With force=False an
    up-to-date library is kept.  stamps=True builds the profiling variant (LIB_STAMPS) instead."""
    if not force and not stamps and not stale():
        return LIB
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    objdir = os.path.join(HERE, "_build", "stamps" if stamps else "lib")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in HIPCC_FLAGS if f != "-shared"] + (["-DSKV_PHASE_STAMPS"] if stamps else [])
    lib = LIB_STAMPS if stamps else LIB
    jobs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src + ".o")
        cmd = [hipcc, *compile_flags, f"-I{INCLUDE}", f"-I{CSRC}", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        jobs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = []
    for src, _, proc in jobs:
        out, _ = proc.communicate()
        if proc.returncode != 0:
            failed.append(f"{src}:\n{out}")
    if failed:
        raise RuntimeError("hipcc failed:\n" + "\n".join(failed))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *[obj for _, obj, _ in jobs], "-o", lib + ".tmp"]
    if verbose:
        print(" ".join(link), flush=True)
    proc = subprocess.run(link, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("link failed:\n" + proc.stdout + proc.stderr)
    os.replace(lib + ".tmp", lib)
    return lib


if __name__ == "__main__":
    import sys
    print(build(force=True, verbose=True, stamps="--stamps" in sys.argv[1:]))
