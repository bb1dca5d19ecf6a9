"""Build the CPU oracle (test infrastructure only) as two shared libraries:
libcgo_f32.so (REAL=float) and libcgo_f64.so (REAL=double)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SOURCES = ["cgo_conv.c", "cgo_layers.c", "cgo_sgd.c"]
FLAGS = ["-O2", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared",
         "-std=c11", "-Wall", "-Wextra", "-Wno-unknown-pragmas"]


def lib_path(real):
    return os.path.join(HERE, "libcgo_f32.so" if real == "float" else "libcgo_f64.so")


def build(force=True):
    for real in ("float", "double"):
        out = lib_path(real)
        srcs = [os.path.join(HERE, s) for s in SOURCES]
        if not force and os.path.exists(out) and all(
                os.path.getmtime(out) >= os.path.getmtime(p) for p in srcs + [os.path.join(HERE, "cgo.h")]):
            continue
        cmd = ["gcc", *FLAGS, f"-DREAL={real}", "-I", HERE, *srcs, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)
    return lib_path("float"), lib_path("double")


if __name__ == "__main__":
    print(*build(force="--if-stale" not in sys.argv), sep="\n")
