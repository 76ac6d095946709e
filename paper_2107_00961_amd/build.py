"""Compile the HIP library (gfx950) in-tree: paper_2107_00961_amd/libresist.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INC = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libresist.so")
OBJ = os.path.join(HERE, "_build")
SOURCES = ["model.cpp", "step.cpp", "ops.cpp", "prof.cpp", "overlap.cpp", "conv.hip", "bn.hip", "head.hip", "stem.hip", "update.hip", "compress.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3"] + os.environ.get("RESIST_EXTRA_FLAGS", "").split() + ["-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-I", INC, "-I", CSRC]


def build(verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    procs = []
    for src in SOURCES:
        obj = os.path.join(OBJ, src + ".o")
        cmd = [hipcc] + FLAGS + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
    objs = []
    for src, obj, p in procs:
        out = p.communicate()[0].decode()
        # hipcc's host pass does not know the packed-fp32 target feature and says so: harmless
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
        objs.append(obj)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


def build_host_check():
    """The library's host-only code (model.cpp) with its driver host_check.cpp under AddressSanitizer and
    UndefinedBehaviorSanitizer, host compiler only: paper_2107_00961_amd/_build/host_check."""
    os.makedirs(OBJ, exist_ok=True)
    exe = os.path.join(OBJ, "host_check")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan", "-Wall", "-D__HIP_PLATFORM_AMD__",
           "-I", "/opt/rocm/include", "-I", INC, "-I", CSRC, "-o", exe,
           os.path.join(CSRC, "host_check.cpp"), os.path.join(CSRC, "model.cpp")]
    subprocess.check_call(cmd)
    return exe


if __name__ == "__main__":
    print(build_host_check() if "--sanitize" in sys.argv else build(verbose="-v" in sys.argv))
