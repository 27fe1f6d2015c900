"""Builds libq8nmt.so (the C-ABI library of HIP kernels) in-tree with hipcc for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libq8nmt.so")
SOURCES = ["q8_products.hip", "q8_gemm.hip", "q8_gru.hip", "q8_decoder.hip", "q8_output.hip", "q8_search.hip", "q8_fp32.hip", "q8_noalloc.hip", "q8_api.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-fPIC", "-shared", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _run(cmd):
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), err))
    return err


def build(verbose=False):
    """Compiles every source to an object (in parallel) and links the shared library."""
    from concurrent.futures import ThreadPoolExecutor
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    compile_flags = [f for f in FLAGS if f != "-shared"]
    objs = [os.path.join(objdir, s.rsplit(".", 1)[0] + ".o") for s in SOURCES]
    cmds = [["hipcc", *compile_flags, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(6, len(cmds))) as ex:
        errs = list(ex.map(_run, cmds))
    errs.append(_run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]))
    if verbose:
        print("\n".join(e for e in errs if e.strip()))
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
