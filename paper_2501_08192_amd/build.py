"""Build libpreserve_mi355x.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpreserve_mi355x.so")
SOURCES = ["gemv.hip", "gemm_sk.hip", "attention.hip", "window.hip", "segment.hip", "step.hip", "static_step.hip", "executor.cpp", "api.cpp", "planner.cpp"]
HEADERS = [os.path.join(CSRC, "internal.h"), os.path.join(CSRC, "device.h"), os.path.join(CSRC, "context.h"), os.path.join(CSRC, "tagged.h"), os.path.join(CSRC, "prefetch.h"),
           os.path.join(HERE, "..", "include", "preserve.h"), os.path.join(HERE, "..", "include", "preserve_aux.h")]

# Packed-FP32 VALU instructions are switched off for all device code.
HIP_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-Wall", "-Wno-unused-result",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def is_stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, s) for s in SOURCES] + HEADERS
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, verbose: bool = False) -> str:
    if not force and not is_stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    def compile_one(s):
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        cmd = [hipcc] + HIP_FLAGS + ["-c", os.path.join(CSRC, s), "-o", obj]
        if s.endswith(".cpp"):
            cmd = [hipcc, "-O2", "-std=c++17", "-fPIC", "-Wall", "-c", os.path.join(CSRC, s), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        return s, obj, r

    objs = []
    with ThreadPoolExecutor(max_workers=min(len(SOURCES), 8)) as pool:      # the files are independent
        results = list(pool.map(compile_one, SOURCES))
    for s, obj, r in results:
        if verbose or r.returncode != 0:
            sys.stderr.write(r.stdout + "\n".join(
                l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l) + "\n")
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on " + s)
        objs.append(obj)
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        sys.stderr.write(r.stdout + r.stderr)
        raise RuntimeError("link failed")
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True))
