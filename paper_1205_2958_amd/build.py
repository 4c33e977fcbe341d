"""Builds libminhash.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_1205_2958_amd.build

hipcc cross-compiles without a GPU.  The shared object lands next to this file
so that it travels with the source tree; nothing is installed.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRCS = [os.path.join(HERE, "csrc", "minhash.hip"), os.path.join(HERE, "csrc", "consumers.hip"),
        os.path.join(HERE, "csrc", "ingest.hip"), os.path.join(HERE, "csrc", "packed.hip")]
LIB = os.path.join(HERE, "libminhash.so")
# measurement only (instruction-issue and memory probes behind bench.py --probe); the signature library does not use it
PROBE_SRCS = [os.path.join(HERE, "csrc", "probe.hip")]
PROBE_LIB = os.path.join(HERE, "libminhash_probe.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared", "-pthread",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc"),
]


def _compile(srcs, lib, verbose, extra) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + list(extra) + srcs + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only target feature; that warning is harmless
    log = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("hipcc failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(tmp, lib)
    return lib


def build(verbose: bool = False, extra=()) -> str:
    """Compiles both libraries (side by side: the probe library takes a tenth of the time of the other);
    returns the path of the signature library."""
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(2) as pool:
        probe = pool.submit(_compile, PROBE_SRCS, PROBE_LIB, verbose, extra)
        main = pool.submit(_compile, SRCS, LIB, verbose, tuple(extra) + ("-parallel-jobs=4",))
        probe.result()
        return main.result()


if __name__ == "__main__":
    print(build(verbose=True, extra=sys.argv[1:]))
