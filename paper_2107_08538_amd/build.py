"""Build libmgb.so (scheduler + HIP task kernels) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmgb.so")
SOURCES = ["sched.cpp", "lazy.cpp", "ipc.cpp", "runner.cpp", "jacobi.hip", "gemm_f32.hip", "gemm_bf16.hip", "conv3x3.hip", "bfs.hip", "cu_trace.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-value", "-Wno-unused-command-line-argument", "-Wno-inline-asm"]


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc"] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    lines = [l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l]
    return src, obj, r.returncode, "\n".join(lines)


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        results = list(ex.map(_compile, srcs))
    objs = []
    for src, obj, rc, log in results:
        if rc != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, log))
        if verbose and log.strip():
            print(log)
        objs.append(obj)
    subprocess.check_call(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-lpthread", "-lrt"])
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
