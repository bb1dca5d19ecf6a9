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
    if src == "igemm.hip":
        cmd.append("-Rpass-analysis=kernel-resource-usage")
    r = subprocess.run(cmd, capture_output=True, text=True)
    if src == "igemm.hip" and r.returncode == 0 and not flags:       # the fp32 build; the bf16 builds use the long forms only
        # The LDS-direct loads of the matrix kernels are inline assembly that reads buffer descriptors
        # from scalar registers.  A scalar register restored from a spill is written by a vector
        # instruction (v_readlane), after which a vector-memory instruction may read it only five wait
        # states later, and nothing checks that inside assembly.  The patch, band and 16-row kernels
        # spill scalar registers (their set-up holds many) and therefore use only the load forms that
        # carry five wait states of their own (s_mov m0 + s_nop 3).  The gathered kernel uses the short
        # forms (one or two wait states), which is safe only while it spills nothing: a build in which
        # it does is refused.
        name, bad = None, []
        for line in r.stderr.splitlines():
            if "Function Name:" in line:
                name = line.split("Function Name:")[1].split()[0]
            elif "SGPRs Spill:" in line and name and "12igemm_kernelI" in name:
                if int(line.split("SGPRs Spill:")[1].split()[0]) != 0:
                    bad.append(name)
        if bad:
            raise RuntimeError("the gathered matrix kernel spills scalar registers (descriptor hazard of its short load forms): " + ", ".join(sorted(set(bad))))

    # the host pass does not know the packed-fp32 feature switch; that warning is harmless.  The
    # resource-usage remarks (and the source lines quoted under them) have been read above.
    import re
    lines = [l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l]
    if src == "igemm.hip":
        lines = [l for l in lines if "remark:" not in l and not re.match(r"^\s*\d*\s*\|", l)]
    err = "\n".join(lines)
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
