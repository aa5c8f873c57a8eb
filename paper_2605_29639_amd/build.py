"""Build the C-ABI library (hand-written HIP for gfx950) into paper_2605_29639_amd/libkvq.so.

`python -m paper_2605_29639_amd.build` or `build()`.  hipcc cross-compiles without a GPU.
"""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libkvq.so")
OBJ_PROF = os.path.join(HERE, "_build", "prof")
LIB_PROF = os.path.join(HERE, "libkvq_prof.so")
SOURCES = ["kvq_api.hip", "kvq_write.hip", "kvq_attn.hip", "kvq_prefill.hip", "kvq_repack.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # Matrix-instruction results stay in ordinary vector registers.  With the 512-register
         # budget of a one-wavefront-per-SIMD kernel the compiler otherwise puts them into
         # accumulation registers, which no vector instruction can address, and copies every
         # logit and (on each rescale) every output accumulator out and back in.
         "-mllvm", "-amdgpu-mfma-vgpr-form",
         "-Wno-unused-command-line-argument"]


def _compile(job):
    src, objdir, defines = job
    obj = os.path.join(objdir, src.replace(".hip", ".o"))
    subprocess.check_call(["hipcc", *FLAGS, *defines, "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def _link(objs, lib):
    tmp = lib + ".tmp%d" % os.getpid()
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, lib)


def build(verbose: bool = False) -> str:
    """libkvq.so (the library) and libkvq_prof.so (the same sources with -DKVQ_PROFILE: the
    measurement switches of include/kvq_prof.h on top)."""
    jobs = []
    for objdir, defines in ((OBJ, []), (OBJ_PROF, ["-DKVQ_PROFILE"])):
        os.makedirs(objdir, exist_ok=True)
        jobs += [(src, objdir, defines) for src in SOURCES]
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, jobs))
    _link(objs[:len(SOURCES)], LIB)
    _link(objs[len(SOURCES):], LIB_PROF)
    if verbose:
        print("built", LIB, "and", LIB_PROF)
    return LIB


if __name__ == "__main__":
    build(verbose=True)
