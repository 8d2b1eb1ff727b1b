"""Builds liblamps.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2410_18248_amd.build

hipcc cross-compiles without a GPU.  Objects go to _build/ (ignored), the
library next to this file so that it travels with the source tree.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblamps.so")
SOURCES = ["decode_attn.hip", "block_copy.hip", "kv_append.hip", "prefill_attn.hip", "lamps.cpp", "sched.cpp"]
# the scheduler's times are compared bit for bit with a plain evaluation of the same formulas:
# no fused multiply-adds in its host code
PER_SOURCE = {"sched.cpp": ["-ffp-contract=off"],
              # the prefill kernel rescales its MFMA accumulators on the vector ALUs now and then;
              # with the accumulators in ordinary vector registers that needs no register moves, and
              # mfma_f32_16x16x32_bf16 issues every 16 cycles instead of every 30-47 (measured); the
              # HBM-bound decode kernels are 2-4 % slower that way (registers) and keep the default
              "prefill_attn.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
         # packed fp32 VALU forms are kept out of the generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def _compile(src, obj, extra):
    cmd = [HIPCC] + FLAGS + PER_SOURCE.get(src, []) + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(verbose=False, extra=(), out=None):
    """Compiles the sources and links `out` (default: liblamps.so next to this file)."""
    lib = out or LIB
    bdir = os.path.join(ROOT, "_build", os.path.basename(lib))
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.rsplit(".", 1)[0] + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        list(ex.map(lambda so: _compile(so[0], so[1], list(extra)), zip(SOURCES, objs)))
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    args = sys.argv[1:]
    out = None
    if "-o" in args:
        i = args.index("-o")
        out = os.path.abspath(args[i + 1])
        del args[i:i + 2]
    build(verbose=True, extra=args, out=out)
