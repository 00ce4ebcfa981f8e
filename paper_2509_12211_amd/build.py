"""Builds libtinyserve_hip.so (gfx950) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtinyserve_hip.so")
# the same sources with phase timestamps compiled in (bench.py --phase-marks); built on request
PROFILE_LIB = os.path.join(HERE, "libtinyserve_prof.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    "-Wno-unused-function", "-Wno-unknown-warning-option",
    # packed-FP32 instruction selection is switched off for all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def stale(lib: str = LIB) -> bool:
    if not os.path.exists(lib):
        return True
    t = os.path.getmtime(lib)
    deps = sources() + glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(
        os.path.join(HERE, "..", "include", "*.h"))
    return any(os.path.getmtime(d) > t for d in deps)


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the packed-fp32 feature and says so: harmless
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out, flush=True)


def build(force: bool = True, verbose: bool = False, profile: bool = False) -> str:
    """Compile every .hip file of csrc/ to an object (in parallel: every cache format and
    head_dim is a file of its own) and link them into the shared library.  profile=True
    builds the tuning library instead: the same code with -DTS_PROFILE, whose fused kernel
    records a timestamp at each numbered point of its path (ts_debug_set_profile_buffer)."""
    lib = PROFILE_LIB if profile else LIB
    if not force and not stale(lib):
        return lib
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build_prof" if profile else "_build")
    flags = HIPCC_FLAGS + (["-DTS_PROFILE"] if profile else [])
    os.makedirs(objdir, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    for stale_obj in set(glob.glob(os.path.join(objdir, "*.o"))) - set(objs):
        os.remove(stale_obj)          # objects of sources that no longer exist
    jobs = min(len(srcs), max(1, min(os.cpu_count() or 1, 8)))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        list(pool.map(lambda so: _run([hipcc] + flags + ["-c", so[0], "-o", so[1]], verbose),
                      zip(srcs, objs)))
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", lib], verbose)
    return lib


if __name__ == "__main__":
    import sys
    print(build(force=True, verbose=True, profile="--profile" in sys.argv))
