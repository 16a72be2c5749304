"""Compile the HIP sources of libvs for gfx950 (MI355X) with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libvs.so")
SOURCES = ["vs_api.hip", "vs_attn.hip", "vs_estimate.hip", "vs_select.hip"]
HEADERS = [os.path.join(CSRC, "vs_common.h"), os.path.join(HERE, "..", "include", "vs.h")]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # packed fp32 VALU forms are switched off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # hardware fp32 atomic add (LDS and global) instead of compare-and-swap loops
    "-munsafe-fp-atomics",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    raise RuntimeError("hipcc not found")


def _stale(target: str, deps: list[str]) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = False, verbose: bool = False, extra_flags: list[str] | None = None,
          variant: str | None = None) -> str:
    """Compile and link libvs.so.  With `variant` the objects go to _build/<variant>/ and the library
    to libvs_<variant>.so next to libvs.so (a build with other -D switches, e.g. the timing diagnostics
    of vs_attn.hip; load it by setting VS_LIB_PATH)."""
    build_dir = os.path.join(BUILD, variant) if variant else BUILD
    lib = os.path.join(HERE, f"libvs_{variant}.so") if variant else LIB
    os.makedirs(build_dir, exist_ok=True)
    hipcc = _hipcc()
    flags = FLAGS + (extra_flags or [])
    jobs = []
    for s in SOURCES:
        src, obj = os.path.join(CSRC, s), os.path.join(build_dir, s + ".o")
        if force or _stale(obj, [src] + HEADERS):
            jobs.append((src, obj))

    def cc(job):
        src, obj = job
        cmd = [hipcc] + flags + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{err}")
        if err.strip() and verbose:
            print(err, file=sys.stderr)

    with ThreadPoolExecutor(max_workers=4) as ex:
        list(ex.map(cc, jobs))
    objs = [os.path.join(build_dir, s + ".o") for s in SOURCES]
    if force or jobs or _stale(lib, objs):
        cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("link failed:\n" + r.stderr)
    return lib


def build_ceiling(force: bool = False) -> str:
    """libvs_ceiling.so: the instruction-mix ceiling kernels of csrc/vs_ceiling.hip (a measurement aid that
    bench_ceiling.py runs; not linked into libvs.so)."""
    src, lib = os.path.join(CSRC, "vs_ceiling.hip"), os.path.join(HERE, "libvs_ceiling.so")
    if force or _stale(lib, [src]):
        cmd = [_hipcc()] + [f for f in FLAGS if f != "-Wall"] + ["-shared", "-o", lib, src]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed for vs_ceiling.hip:\n" + r.stderr)
    return lib


if __name__ == "__main__":
    # python -m paper_2501_15383_amd.build [--force] [--variant NAME -DSWITCH ...]
    argv = sys.argv[1:]
    var = argv[argv.index("--variant") + 1] if "--variant" in argv else None
    print(build(force="--force" in argv, verbose=True, variant=var,
                extra_flags=[a for a in argv if a.startswith("-D")]))
