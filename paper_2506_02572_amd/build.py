"""Build libhata.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libhata.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["hata_api.hip", "hata_encode.hip", "hata_score.hip", "hata_topk.hip", "hata_attn.hip", "hata_gather.hip", "hata_coop.hip",
           "hata_train.hip", "hata_probe.hip"]
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
    if trace:
        cmds = [[HIPCC] + FLAGS + ["-DHATA_TRACE", "-fgpu-rdc"] + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]]
        link = None
    else:
        # one object per source, compiled side by side (objects of sources that did not change are
        # kept unless force is set), then one link
        os.makedirs(OBJ, exist_ok=True)
        newest_header = max(os.path.getmtime(os.path.join(CSRC, h)) for h in HEADERS)
        compile_flags = [f for f in FLAGS if f != "-shared"] + ["-c"]
        cmds, objs = [], []
        for src in SOURCES:
            o = os.path.join(OBJ, src.replace(".hip", ".o"))
            objs.append(o)
            fresh = os.path.exists(o) and os.path.getmtime(o) > max(newest_header, os.path.getmtime(os.path.join(CSRC, src)))
            if force or not fresh:
                cmds.append([HIPCC] + compile_flags + [os.path.join(CSRC, src), "-o", o])
        link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB]

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out)

    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(8, max(1, len(cmds)))) as pool:
        list(pool.map(run, cmds))
    if link:
        run(link)
    return LIB


if __name__ == "__main__":
    build(force="--changed" not in sys.argv, verbose=True, trace="--trace" in sys.argv)
    print(LIB)
