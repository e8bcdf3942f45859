"""Build libthanos.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2504_05346_amd.build            # incremental
    python -m paper_2504_05346_amd.build --force    # recompile everything
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libthanos.so")
SOURCES = ["api.hip", "syrk.hip", "gemm_f32.hip", "factor.hip", "sweep.hip", "structured.hip"]
HEADERS = ["common.h", "gemm_tile.h", "gemm_tile_x3.h", "timeline.h",
           os.path.join("..", "..", "include", "thanos.h")]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def _stale(target: str, deps: list[str]) -> bool:
    if not os.path.exists(target):
        return True
    t = os.path.getmtime(target)
    return any(os.path.getmtime(d) > t for d in deps)


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ, src.replace(".hip", ".o"))
    deps = [os.path.join(CSRC, src)] + [os.path.join(CSRC, h) for h in HEADERS]
    if force or _stale(obj, deps):
        cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
        if r.stderr.strip():
            sys.stderr.write(r.stderr)
    return obj


PROBE_SRC = os.path.join(CSRC, "probe", "peak_probe.hip")
PROBE_LIB = os.path.join(HERE, "libthanos_probe.so")


def build_probe(force: bool = False) -> str:
    """libthanos_probe.so: stand-alone microbenchmarks (measured matrix-core and HBM ceilings)."""
    if force or _stale(PROBE_LIB, [PROBE_SRC]):
        cmd = [HIPCC, *FLAGS, "-shared", PROBE_SRC, "-o", PROBE_LIB]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for the probe:\n{r.stdout}\n{r.stderr}")
    return PROBE_LIB


TIMELINE_LIB = os.path.join(HERE, "libthanos_timeline.so")


def _compile_timeline(force: bool) -> str:
    """sweep.hip once more with -DTHANOS_TIMELINE (timestamps inside k_update, see timeline.h)."""
    obj = os.path.join(OBJ, "sweep_timeline.o")
    deps = [os.path.join(CSRC, "sweep.hip")] + [os.path.join(CSRC, h) for h in HEADERS]
    if force or _stale(obj, deps):
        cmd = [HIPCC, *FLAGS, "-DTHANOS_TIMELINE", "-c", os.path.join(CSRC, "sweep.hip"), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for the timeline build:\n{r.stdout}\n{r.stderr}")
    return obj


def _link(lib: str, objs: list[str], force: bool) -> None:
    if force or _stale(lib, objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")


def build(force: bool = False) -> str:
    """libthanos.so (the product), libthanos_probe.so (peak probe) and libthanos_timeline.so (the
    product's sources with the timestamps of timeline.h compiled in; used by timeline_probe.py
    only)."""
    os.makedirs(OBJ, exist_ok=True)
    build_probe(force)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES) + 1)) as ex:
        tl = ex.submit(_compile_timeline, force)
        objs = list(ex.map(lambda s: _compile(s, force), SOURCES))
        tl_obj = tl.result()
    _link(LIB, objs, force)
    sweep_obj = os.path.join(OBJ, "sweep.o")
    _link(TIMELINE_LIB, [tl_obj if o == sweep_obj else o for o in objs], force)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
