"""Compile the C oracle with gcc: fp64 reference and fp32 diagnostic mirror.

TEST INFRASTRUCTURE ONLY (see oracle/cocod_oracle.c).  Run as a script or call build().
"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "cocod_oracle.c")
LIBS = {"f64": ("liboracle_f64.so", "double"), "f32": ("liboracle_f32.so", "float")}


def lib_path(kind="f64"):
    return os.path.join(HERE, LIBS[kind][0])


def build(force=True):
    for kind, (name, real) in LIBS.items():
        out = os.path.join(HERE, name)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
            continue
        # -ffp-contract=off: every product and sum is rounded on its own, as written
        cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-DREAL=" + real, SRC, "-o", out, "-lm"]
        subprocess.run(cmd, check=True)


if __name__ == "__main__":
    build()
    print("built", [lib_path(k) for k in LIBS])
