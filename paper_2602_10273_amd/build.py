"""Build libpower_smc.so (HIP, gfx950 only) in-tree with hipcc.  No JIT, no torch extension machinery.

Every translation unit is compiled to an object of its own (in parallel) and the objects are linked into the
shared library.  build() recompiles everything; build(incremental=True) only what is older than its sources.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpower_smc.so")
SOURCES = ["smc_api.hip", "vocab_pass_bf16.hip", "vocab_pass_f32.hip", "vocab_pass.hip", "weights.hip", "kv_gather.hip", "paged_kv.hip", "hbm_probe.hip",
           "attn_decode.hip", "kv_append.hip", "noalloc.hip"]
HEADERS = ["smc_internal.hpp", "device_rng.hpp", "weights_device.hpp", "gather_plan_device.hpp", "vocab_pass_kernel.hpp", os.path.join(ROOT, "include", "power_smc.h")]

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _header_paths():
    return [h if os.path.isabs(h) else os.path.join(CSRC, h) for h in HEADERS]


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + _header_paths()
    return any(os.path.getmtime(d) > t for d in deps)


def build(verbose: bool = False, incremental: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(h) for h in _header_paths())

    def compile_one(src):
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, src.replace(".hip", ".o"))
        if incremental and os.path.exists(o) and os.path.getmtime(o) >= max(os.path.getmtime(s), newest_header):
            return o
        cmd = [hipcc] + FLAGS + ["-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return o

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))
