"""Builds libcomet_hip.so (all HIP sources, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libcomet_hip.so")
OBJ_DIR = os.path.join(_HERE, "_build")

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
               # packed-fp32 VALU forms are kept out of the generated code on purpose
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-result"]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False, only_changed: bool = False) -> str:
    """Compile every HIP source (one hipcc process per file, side by side) and link them into one
    shared library.  Always recompiles everything unless only_changed is set (development aid:
    then a source is recompiled when it or any header is newer than its object file)."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(_HERE, "..", "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs = []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        fresh = (only_changed and os.path.exists(obj)
                 and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            jobs.append([hipcc, *HIPCC_FLAGS, "-c", "-o", obj, src])
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        list(pool.map(lambda c: _run(c, verbose), jobs))
    tmp = LIB_PATH + ".tmp%d" % os.getpid()
    objs = [os.path.join(OBJ_DIR, os.path.basename(src) + ".o") for src in sources()]
    _run([hipcc, "--offload-arch=gfx950", "-fPIC", "-shared", "-o", tmp, *objs], verbose)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def build_if_missing() -> str:
    """The built library if there is one (tests, the smoke check and the benchmark load what is built), else
    build it.  A library older than a source or header is still used -- the build step is explicit -- but
    that is said loudly, since results then come from stale code."""
    if os.path.exists(LIB_PATH):
        deps = sources() + glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(_HERE, "..", "include", "*.h"))
        newest = max(deps, key=os.path.getmtime)
        if os.path.getmtime(LIB_PATH) < os.path.getmtime(newest):
            import sys
            print("WARNING: %s is older than %s -- run `python -m paper_2102_05187_amd.build` to rebuild" % (
                os.path.basename(LIB_PATH), os.path.relpath(newest, _HERE)), file=sys.stderr, flush=True)
        return LIB_PATH
    return build()


if __name__ == "__main__":
    import sys
    print(build(verbose=True, only_changed="--changed" in sys.argv))
