"""Builds libspecpv.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libspecpv.so")
# the same library with time stamps inside the partial-verify attention kernel (timeline.py uses it)
LIB_TIMELINE = os.path.join(HERE, "libspecpv_timeline.so")
SOURCES = ["api.hip", "summarize.hip", "select.hip", "score_mfma.hip", "attn_generic.hip",
           "attn_mfma.hip", "combine.hip", "commit.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # leading scalar kernel arguments arrive in registers instead of through a load
         "-mllvm", "-amdgpu-kernarg-preload-count=12",
         "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build(verbose=False, jobs=8, lib=LIB, defines=()):
    """Compile every HIP source to an object (in parallel) and link the shared library `lib`."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("SPECPV_EXTRA_HIPCC_FLAGS", "").split() + ["-D" + d for d in defines]
    objdir = os.path.join(HERE, "_build", os.path.basename(lib).replace(".so", ""))
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            procs[0][1].wait() if procs[0][1].poll() is None else None
            for _, p in procs:
                if p.poll() is None:
                    p.wait()
                    break
    for src, p in procs:
        out, _ = p.communicate()
        # the host pass does not know the packed-fp32 target feature and says so: harmless
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs, check=True)
    os.replace(tmp, lib)
    return lib


def build_timeline(verbose=False):
    """The instrumented variant: same sources, -DSPECPV_TIMELINE, its own file name."""
    return build(verbose=verbose, lib=LIB_TIMELINE, defines=("SPECPV_TIMELINE",))


if __name__ == "__main__":
    import sys
    print(build_timeline(verbose=True) if "--timeline" in sys.argv[1:] else build(verbose=True))
