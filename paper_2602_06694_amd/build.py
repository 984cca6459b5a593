"""Build libnq_binlr.so (HIP, gfx950) in-tree with hipcc.

    python -m paper_2602_06694_amd.build [--changed]     (--changed: recompile only sources older than their object)

The library is placed next to this file so that it travels with the source
tree; nothing is installed.  The C-ABI header lives in ``include/``.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libnq_binlr.so")
SOURCES = ["nq_api.hip", "nq_admm.hip", "nq_decode.hip", "nq_exec.hip", "nq_prefill.hip", "nq_probe.hip", "nq_transposed.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 instructions are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return [os.path.join(CSRC, s) for s in SOURCES]


HEADERS = [os.path.join(CSRC, "nq_internal.h"), os.path.join(CSRC, "nq_device.h"), os.path.join(ROOT, "include", "nq_binlr.h"),
           os.path.join(ROOT, "include", "nq_lb_admm.h")]
OBJ_DIR = os.path.join(HERE, "_build")


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(d) > t for d in sources() + HEADERS)


# per-source additions: the matrix-core probe loops keep their accumulators in ordinary vector registers (left to itself
# the compiler moves them between the two register files in every iteration of those loops)
EXTRA_FLAGS = {"nq_probe.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _compile_one(src: str, obj: str, verbose: bool) -> str:
    cmd = [HIPCC] + [f for f in FLAGS if f != "-shared"] + EXTRA_FLAGS.get(os.path.basename(src), []) + ["-c", src, "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the device-only feature flag; that warning is noise
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {os.path.basename(src)}:\n{err}")
    return err


def build(force: bool = True, verbose: bool = False) -> str:
    """Compiles every source to an object of its own (in parallel; with force=False only those older than their
    source or a header) and links the shared library."""
    if not force and not is_stale():
        return LIB
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJ_DIR, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in HEADERS)
    jobs, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src) + ".o")
        objs.append(obj)
        fresh = os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header)
        if force or not fresh:
            jobs.append((src, obj))
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(jobs)))) as pool:
        for err in pool.map(lambda j: _compile_one(j[0], j[1], verbose), jobs):
            if err.strip():
                sys.stderr.write(err + "\n")
    tmp = LIB + f".tmp{os.getpid()}"
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr + "\n")
        raise RuntimeError("hipcc failed linking libnq_binlr.so")
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force="--changed" not in sys.argv, verbose=True))
