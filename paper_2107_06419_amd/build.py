"""Build the HIP libraries in-tree (gfx950 only): paper_2107_06419_amd/libflat_attn.so, its fully synchronised
checking build libflat_attn_sync.so, and the measurement aids libflat_attn_probe.so."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libflat_attn.so")
SOURCES = ["flat_api.hip", "flat_fwd_bf16.hip", "flat_fwd_bf16_shapes_d64a.hip", "flat_fwd_bf16_shapes_d64b.hip",
           "flat_fwd_bf16_shapes_d64c.hip", "flat_fwd_bf16_shapes_d128.hip", "flat_fwd_bf16_shapes_dx.hip", "flat_splitkv.hip", "flat_plan.hip", "flat_tiles.hip", "flat_fwd_f32.hip", "flat_unfused.hip"]
# the measurement aids live in a library of their own
PROBE_LIB = os.path.join(HERE, "libflat_attn_probe.so")
PROBE_SOURCES = ["flat_probe.hip", "flat_probe_api.hip"]
# packed fp32 VALU instructions are switched off for all device code
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


# Checking build: the fused bf16 kernels with every ring phase fully synchronised (FLAT_SYNC_EVERY_PHASE), linked
# with the unchanged remaining objects into a second library that a GPU test compares bit for bit with the first.
SYNC_LIB = os.path.join(HERE, "libflat_attn_sync.so")
SYNC_SOURCES = [s for s in SOURCES if s.startswith("flat_fwd_bf16") or s == "flat_splitkv.hip"]


def _compile(src: str, sync: bool = False) -> str:
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + (".sync.o" if sync else ".o"))
    cmd = [_hipcc(), *FLAGS, *(["-DFLAT_SYNC_EVERY_PHASE"] if sync else []), "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build_library(verbose: bool = True) -> str:
    """Compile every kernel source for gfx950 and link the shared library. Always recompiles."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as pool:
        jobs = ([pool.submit(_compile, s) for s in SOURCES] + [pool.submit(_compile, s, True) for s in SYNC_SOURCES] +
                [pool.submit(_compile, s) for s in PROBE_SOURCES])
        objs = [j.result() for j in jobs]
    plain, sync = objs[:len(SOURCES)], objs[len(SOURCES):len(SOURCES) + len(SYNC_SOURCES)]
    probe = objs[len(SOURCES) + len(SYNC_SOURCES):]
    sync_objs = [o for s, o in zip(SOURCES, plain) if s not in SYNC_SOURCES] + sync
    for lib, parts in ((LIB, plain), (SYNC_LIB, sync_objs), (PROBE_LIB, probe)):
        tmp = lib + f".tmp{os.getpid()}"
        subprocess.check_call([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *parts])
        os.replace(tmp, lib)
        if verbose:
            print(f"built {lib}")
    return LIB


if __name__ == "__main__":
    build_library()
