"""Build libhata.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhata.so")
SOURCES = ["hata_api.hip", "hata_encode.hip", "hata_score.hip", "hata_topk.hip", "hata_attn.hip", "hata_coop.hip",
           "hata_train.hip"]
HEADERS = ["hata_device.h", "hata_internal.h", "hata_select.h", "hata_trace.h", "hata_attn_core.h", os.path.join("..", "..", "include", "hata.h"),
           os.path.join("..", "..", "include", "hata_train.h")]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False, trace: bool = False) -> str:
    """trace=True adds the in-kernel timestamp hooks of hata_trace.h (tuning builds only)."""
    if not force and not stale():
        return LIB
    extra = ["-DHATA_TRACE", "-fgpu-rdc"] if trace else []
    cmd = [HIPCC] + FLAGS + extra + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    build(force=True, verbose=True, trace="--trace" in sys.argv)
    print(LIB)
