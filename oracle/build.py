"""Compile oracle/layers.c twice with gcc: REAL=float and REAL=double."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path(real):
    return os.path.join(HERE, "liboracle_%s.so" % ("f32" if real == "float" else "f64"))


def build(force=True):
    src = os.path.join(HERE, "layers.c")
    for real in ("float", "double"):
        out = lib_path(real)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
            continue
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c11",
                               "-DREAL=" + real, src, "-o", out, "-lm"])


if __name__ == "__main__":
    build()
