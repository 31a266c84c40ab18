"""Builds libdetox.so (HIP, gfx950 only) in-tree: one object per translation unit, compiled in
parallel, then linked into paper_1907_12205_amd/libdetox.so."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdetox.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


SORTNET_PARTS = 8      # must equal kSortnetParts in csrc/sortnet.hip
MAX_R = 11             # must equal kMaxR in csrc/detox_internal.h


def units():
    """(source, object name, extra flags): sortnet.hip is compiled once per part plus once bare."""
    out = []
    for src in sources():
        out.append((src, src[:-4] + ".o", []))
        if src == "sortnet.hip":
            for k in range(SORTNET_PARTS):
                out.append((src, f"sortnet_part{k}.o", [f"-DDETOX_SORTNET_PART={k}"]))
        if src == "filter.hip":
            for r in range(1, MAX_R + 1):
                out.append((src, f"filter_r{r}.o", [f"-DDETOX_FILTER_R={r}"]))
    # longest first
    out.sort(key=lambda u: 0 if ("part" in u[1] or "filter_r" in u[1]) else 1)
    return out


def _stale(obj: str, src: str) -> bool:
    """An object is stale when its source, any header it included when it was last compiled (the
    compiler's dependency file beside it; without one: every header) or this file is newer."""
    if not os.path.exists(obj):
        return True
    t = os.path.getmtime(obj)
    deps = [os.path.join(CSRC, src), __file__]
    try:
        text = open(obj[:-2] + ".d").read().replace("\\\n", " ")
        deps += [w for w in text.split()[1:] if not w.startswith("/opt/") and not w.startswith("/usr/")]
    except OSError:
        deps += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if not f.endswith(".hip")]
        deps.append(os.path.join(HERE, "..", "include", "detox.h"))
    return any((not os.path.exists(d)) or os.path.getmtime(d) > t for d in deps)


def _compile(unit, force=True) -> str:
    src, objname, extra = unit
    obj = os.path.join(OBJ, objname)
    if not force and not _stale(obj, src):
        return obj
    cmd = [HIPCC, *FLAGS, *extra, "-MD", "-MF", obj[:-2] + ".d", "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    out = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                    if "packed-fp32-ops" not in l)       # the host pass does not know the feature
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{out}")
    if out.strip():
        print(out, file=sys.stderr)
    return obj


def build(jobs: int = 8, force: bool = True) -> str:
    """force=False recompiles only objects older than any source (development convenience)."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda u: _compile(u, force), units()))
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout + r.stderr)
    build_example()
    return LIB


EXAMPLES = ["detox_step_main", "detox_calls_main"]


def build_example() -> list:
    """The C-ABI-only callers under examples/ (HIP runtime + libdetox.so, no Python, no torch)."""
    out = []
    for name in EXAMPLES:
        src = os.path.join(HERE, "..", "examples", name + ".cpp")
        exe = os.path.join(HERE, "..", "examples", name)
        cmd = [HIPCC, "-O2", "-std=c++17", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include", src,
               "-o", exe, "-L" + HERE, "-ldetox", "-L/opt/rocm/lib", "-lamdhip64",
               "-Wl,-rpath," + HERE, "-Wl,-rpath,/opt/rocm/lib"]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"building the example {name} failed:\n" + r.stdout + r.stderr)
        out.append(exe)
    return out


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))
