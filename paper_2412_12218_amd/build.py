"""Compile the HIP sources under csrc/ into paper_2412_12218_amd/libftc.so for gfx950."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libftc.so")
SRC_DIR = os.path.join(HERE, "csrc")

FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
         "-I" + os.path.join(ROOT, "include"), "-I" + SRC_DIR]


def sources():
    return sorted(glob.glob(os.path.join(SRC_DIR, "*.hip")))


def build(verbose=False, extra_flags=()):
    """Always recompiles; returns the path of the shared library."""
    obj_dir = os.path.join(HERE, "_build")
    os.makedirs(obj_dir, exist_ok=True)
    procs = []
    objs = []
    compile_flags = [f for f in FLAGS if f != "-shared"] + list(extra_flags)
    for src in sources():
        obj = os.path.join(obj_dir, os.path.basename(src) + ".o")
        objs.append(obj)
        cmd = ["hipcc", "-c", *compile_flags, "-o", obj, src]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
    for src, p in procs:
        _, err = p.communicate()
        # the host pass warns that it does not know the packed-fp32 feature; that is harmless
        err = "\n".join(ln for ln in err.splitlines() if "packed-fp32-ops" not in ln)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err)
    subprocess.run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


if __name__ == "__main__":
    import sys
    print(build(verbose=False, extra_flags=sys.argv[1:]))
