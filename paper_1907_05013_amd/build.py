"""Compile the HIP library for gfx950: python -m paper_1907_05013_amd.build"""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpooch.so")
PROBE = os.path.join(HERE, "hbm_copy_probe.bin")
SOURCES = ["pooch.hip", "plan.cpp", "conv.hip", "bn_elt.hip", "pool_loss.hip"]
# packed fp32 instructions are switched off on purpose (the compiler would otherwise form
# v_pk_*_f32 from ordinary float code)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]


def build(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB])
    for o in objs:
        os.remove(o)
    return LIB


def build_probe():
    """the counter-calibration aid (a plain copy kernel of known size, csrc/hbm_copy_probe.hip): not part of the library,
    built only by `python -m paper_1907_05013_amd.build probe` before a `rocprofv3 --pmc` calibration run"""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", os.path.join(CSRC, "hbm_copy_probe.hip"), "-o", PROBE])
    return PROBE


if __name__ == "__main__":
    import sys
    print(build_probe() if sys.argv[1:] == ["probe"] else build(verbose=True))
