"""Compile libsvdcache.so (HIP, gfx950) in-tree.  `python -m paper_2601_07396_amd.build`."""
from __future__ import annotations

import glob
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libsvdcache.so")
PROBES_LIB_PATH = os.path.join(PKG_DIR, "libsvdcache_probes.so")   # memory-system probes for the benchmark only

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # keep the compiler from forming packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # float / double atomicAdd as hardware atomics
    "-munsafe-fp-atomics",
    # the row tiles are register resident, so their loops must unroll completely however long they get
    "-mllvm", "-pragma-unroll-threshold=1000000",
    "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False) -> str:
    srcs = sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "*.hip")))
    if not srcs:
        raise RuntimeError("no HIP sources found")
    obj_dir = os.path.join(PKG_DIR, "_build")
    os.makedirs(obj_dir, exist_ok=True)

    def run(cmd):
        if verbose:
            print(" ".join(cmd), flush=True)
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed:\n" + out)
        if verbose and out.strip():
            print(out)

    # one translation unit per source, compiled side by side, then linked
    objs = [os.path.join(obj_dir, os.path.basename(src)[:-4] + ".o") for src in srcs]
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=min(len(srcs), os.cpu_count() or 1, 8)) as pool:
        list(pool.map(lambda so: run(["hipcc", *HIPCC_FLAGS, "-c", "-o", so[1], so[0]]), zip(srcs, objs)))
    run(["hipcc", "--offload-arch=gfx950", "-fPIC", "-shared", "-o", LIB_PATH, *objs])
    probe_srcs = sorted(glob.glob(os.path.join(PKG_DIR, "csrc", "probes", "*.hip")))
    run(["hipcc", *HIPCC_FLAGS, "-shared", "-o", PROBES_LIB_PATH, *probe_srcs])
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)
