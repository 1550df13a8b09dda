"""Builds libgptq_w4a16.so for gfx950 with hipcc, in-tree.

    python -m paper_2511_19438_amd.build

The kernels are split over several translation units (one per batch size of the vector kernel
and one per tile shape of the MFMA kernel) that compile in parallel; objects go to
``paper_2511_19438_amd/_build`` and the library to ``paper_2511_19438_amd/lib``.
"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_DIR = os.path.join(HERE, "lib")
LIB_PATH = os.path.join(LIB_DIR, "libgptq_w4a16.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
ARCH = "gfx950"
# -packed-fp32-ops: keep the compiler from forming packed fp32 instructions (v_pk_*_f32)
COMMON = ["--offload-arch=" + ARCH, "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc", "-fvisibility=hidden",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-Wall", "-Wno-unused-function"]

DECODE_BATCHES = (1, 2, 4, 8, 16)
PREFILL_TILES = (1, 3, 5, 8)


def units():
    """(source, object name, extra defines) of every translation unit."""
    out = [("gptq_w4a16.hip", "gptq_w4a16.o", []),
           ("unpack_dequant.hip", "unpack_dequant.o", []),
           ("decode.hip", "decode.o", []),
           ("prefill.hip", "prefill.o", []),
           ("skinny.hip", "skinny.o", []),
           ("mid.hip", "mid.o", []),
           ("act_order.hip", "act_order.o", []),
           ("probe.hip", "probe.o", [])]
    for mb in DECODE_BATCHES:
        out.append(("decode_mb.hip", f"decode_mb{mb}.o", [f"-DGPTQ_DECODE_MB={mb}"]))
    for t in PREFILL_TILES:
        out.append(("prefill_tile.hip", f"prefill_tile{t}.o", [f"-DGPTQ_PREFILL_TILE={t}"]))
    return out


def _compile(unit, extra_flags):
    src, obj, defines = unit
    cmd = [HIPCC, *COMMON, *extra_flags, *defines, "-c", os.path.join(CSRC, src), "-o", os.path.join(OBJ_DIR, obj)]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    return unit, proc


def build(verbose: bool = False, jobs: int = 8, extra_flags=()) -> str:
    """Compile every translation unit and link the shared library.  Returns its path."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    os.makedirs(LIB_DIR, exist_ok=True)
    todo = units()
    failed = False
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        for unit, proc in pool.map(lambda u: _compile(u, list(extra_flags)), todo):
            text = (proc.stdout + proc.stderr).strip()
            # the host pass does not know the device-only target feature; that warning is harmless
            text = "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)
            if proc.returncode != 0:
                failed = True
                print(f"[build] FAILED {unit[1]}\n{text}", file=sys.stderr)
            elif verbose and text:
                print(f"[build] {unit[1]}\n{text}")
    if failed:
        raise RuntimeError("hipcc failed")
    objs = [os.path.join(OBJ_DIR, u[1]) for u in todo]
    link = [HIPCC, "--offload-arch=" + ARCH, "-shared", "-fPIC", "-fno-gpu-rdc", "-fvisibility=hidden", "-o", LIB_PATH, *objs]
    subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
