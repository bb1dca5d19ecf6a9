"""Builds libcg.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libcg.so")
# (source, object name, extra flags): igemm.hip is compiled once per arithmetic of the matrix instructions
SOURCES = [("api.hip", "api.o", []), ("igemm.hip", "igemm.o", []), ("igemm.hip", "igemm_bf16.o", ["-DCG_MATH=1"]),
           ("igemm.hip", "igemm_bf16x3.o", ["-DCG_MATH=2"]), ("conv.hip", "conv.o", []), ("sgd.hip", "sgd.o", []),
           ("layers.hip", "layers.o", []), ("net.hip", "net.o", [])]
COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# the update kernel's operation order is its rounding order: no fused multiply-add there
PER_FILE = {"sgd.hip": ["-ffp-contract=off"]}
EXTRA = os.environ.get("CG_EXTRA_FLAGS", "").split()
LIB = os.environ.get("CG_LIB_OUT", LIB)


def _compile(job):
    src, objname, flags = job
    obj = os.path.join(OBJ, objname)
    cmd = ["hipcc", *COMMON, *EXTRA, *PER_FILE.get(src, []), *flags, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass does not know the packed-fp32 feature switch; that warning is harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
    if r.returncode:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stderr}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(jobs=8):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB], check=True)
    return LIB


if __name__ == "__main__":
    print(build())
