"""Build libdmath.so (the C-ABI library of include/dmath.h) for gfx950 with hipcc.

One object per tile configuration, one each for the FP16-input and the FP64 kernels, plus the API object, compiled in parallel, linked in-tree
into ``paper_1604_01416_amd/libdmath.so``.  hipcc cross-compiles without a GPU.
Run as ``python -m paper_1604_01416_amd.build``.
"""
import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdmath.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -packed-fp32-ops off: the compiler must not form packed FP32 instructions on its own.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def num_configs() -> int:
    text = open(os.path.join(CSRC, "configs.h")).read()
    return int(re.search(r"constexpr int kNumCfg = (\d+);", text).group(1))


def _compile(job):
    src, obj, extra = job
    cmd = [HIPCC] + FLAGS + extra + ["-c", src, "-o", obj]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    return cmd, res.returncode, res.stdout


def sources_newer_than(path: str) -> bool:
    if not os.path.exists(path):
        return True
    t = os.path.getmtime(path)
    for root in (CSRC, os.path.join(os.path.dirname(HERE), "include")):
        for f in os.listdir(root):
            if os.path.getmtime(os.path.join(root, f)) > t:
                return True
    return False


def build(force: bool = True, jobs: int = 8, verbose: bool = False) -> str:
    if not force and not sources_newer_than(LIB):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    work = [(os.path.join(CSRC, "dmath_api.hip"), os.path.join(OBJ, "dmath_api.o"), []),
            (os.path.join(CSRC, "hgemm_instance.hip"), os.path.join(OBJ, "hgemm_instance.o"), []),
            (os.path.join(CSRC, "dgemm_instance.hip"), os.path.join(OBJ, "dgemm_instance.o"), []),
            (os.path.join(CSRC, "wavek_instance.hip"), os.path.join(OBJ, "wavek_instance.o"), [])]
    for i in range(num_configs()):
        work.append((os.path.join(CSRC, "tile_instance.hip"), os.path.join(OBJ, "tile_%d.o" % i),
                     ["-DDMATH_CFG_INDEX=%d" % i]))
    with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(work)))) as pool:
        for cmd, rc, out in pool.map(_compile, work):
            # hipcc's host pass does not know the packed-fp32 feature name; that warning is harmless
            out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
            if verbose or rc != 0:
                sys.stderr.write(" ".join(cmd) + "\n" + out + "\n")
            if rc != 0:
                raise RuntimeError("hipcc failed: " + " ".join(cmd))
    tmp = LIB + ".tmp.%d" % os.getpid()
    link = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + [w[1] for w in work]
    subprocess.check_call(link)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
