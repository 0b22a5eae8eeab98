"""Builds libziplm.so (hand-written HIP for gfx950) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libziplm.so")
SOURCES = ["api.hip", "hessian.hip", "hinv.hip", "prune.hip", "prune_lazy.hip", "prior.hip", "search.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I" + INCLUDE, "-I" + CSRC,
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
# hinv.hip keeps 64-entry rows in registers inside doubly nested, fully unrolled loops; past the default size limit
# of "#pragma unroll" the compiler would leave the outer loop rolled and put those rows in scratch memory
# prune_lazy.hip: its LDS atomics are issued by one lane on purpose; the compiler's wave-level rewrite of atomic adds
# (lane count, one atomic, broadcast) puts a wait and a dozen instructions on the step's critical chain
FILE_FLAGS = {"hinv.hip": ["-mllvm", "-pragma-unroll-threshold=1000000"],
              "prune_lazy.hip": ["-mllvm", "-amdgpu-atomic-optimizer-strategy=None"]}


def build(verbose=False):
    """Compiles csrc/*.hip and links libziplm.so next to this file.

    Environment (optional): HIPCC; ZIPLM_EXTRA_HIPCC_FLAGS, e.g. "-DZIPLM_LAZY_TIMING" for the build that
    prints the greedy loop's per-phase times; ZIPLM_BUILD_LIB, another output path for such a build (its
    objects then go to a directory beside it, so the regular build is left alone)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("ZIPLM_EXTRA_HIPCC_FLAGS", "").split()
    lib = os.environ.get("ZIPLM_BUILD_LIB") or LIB
    objdir = CSRC if lib == LIB else lib + ".objs"
    os.makedirs(objdir, exist_ok=True)
    objs = []
    procs = []
    for s in SOURCES:
        obj = os.path.join(objdir, os.path.splitext(s)[0] + ".o")
        cmd = [hipcc] + FLAGS + FILE_FLAGS.get(s, []) + extra + ["-c", os.path.join(CSRC, s), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for s, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (s, out))
        if verbose and out.strip():
            print(out)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
