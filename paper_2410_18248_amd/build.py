"""Builds liblamps.so (HIP kernels + C ABI) for gfx950, in-tree.

    python -m paper_2410_18248_amd.build

hipcc cross-compiles without a GPU.  Objects go to _build/ (ignored), the
library next to this file so that it travels with the source tree.

Sanitizer build of the host code (for the CPU container; GPU code is not
instrumented):

    LAMPS_SANITIZE=1 python -m paper_2410_18248_amd.build
    LAMPS_SANITIZE=1 python -m paper_2410_18248_amd.build --run python -m pytest tests -q -m "not gpu"

The first line builds _build/sanitize/liblamps.so (and the oracle's C file the
same way) with AddressSanitizer and UndefinedBehaviorSanitizer on the host side
of every source; the second runs a command with that library selected and the
sanitizer's runtime loaded first (a Python process has to preload it).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblamps.so")
SOURCES = ["decode_attn.hip", "block_copy.hip", "kv_append.hip", "prefill_attn.hip", "validate.hip", "lamps.cpp",
           "sched.cpp"]
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


SANITIZE = os.environ.get("LAMPS_SANITIZE", "") not in ("", "0")
SAN_DIR = os.path.join(ROOT, "_build", "sanitize")
# host side only: each -fsanitize= directly behind -Xarch_host
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]


def asan_runtime():
    """The shared AddressSanitizer runtime of the compiler hipcc drives."""
    out = subprocess.check_output([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    if not os.path.isabs(out):
        import glob
        hits = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        out = hits[0] if hits else out
    return out


def _compile(src, obj, extra):
    cmd = [HIPCC] + FLAGS + PER_SOURCE.get(src, []) + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    subprocess.check_call(cmd)
    return obj


def build(verbose=False, extra=(), out=None):
    """Compiles the sources and links `out` (default: liblamps.so next to this file)."""
    san = SANITIZE and out is None
    if san:
        os.makedirs(SAN_DIR, exist_ok=True)
        extra = list(extra) + SAN_FLAGS
    lib = out or (os.path.join(SAN_DIR, "liblamps.so") if san else LIB)
    bdir = os.path.join(ROOT, "_build", ("san-" if san else "") + os.path.basename(lib))
    os.makedirs(bdir, exist_ok=True)
    objs = [os.path.join(bdir, s.rsplit(".", 1)[0] + ".o") for s in SOURCES]
    with ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
        list(ex.map(lambda so: _compile(so[0], so[1], list(extra)), zip(SOURCES, objs)))
    link = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libasan"] if san else []
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + link + objs)
    if verbose:
        print("built", lib)
    return lib


def run_sanitized(cmd):
    """Runs cmd with the sanitized libraries selected and the sanitizer runtime preloaded."""
    env = dict(os.environ, LAMPS_SANITIZE="1")
    pre = [asan_runtime()] + [x for x in env.get("LD_PRELOAD", "").split(":") if x]
    env["LD_PRELOAD"] = ":".join(pre)
    # Python and numpy are not instrumented and never free some of what they allocate
    env.setdefault("ASAN_OPTIONS", "detect_leaks=0:verify_asan_link_order=0")
    env.setdefault("UBSAN_OPTIONS", "print_stacktrace=1:halt_on_error=1")
    return subprocess.call(cmd, env=env)


if __name__ == "__main__":
    args = sys.argv[1:]
    if "--run" in args:
        i = args.index("--run")
        sys.exit(run_sanitized(args[i + 1:]))
    out = None
    if "-o" in args:
        i = args.index("-o")
        out = os.path.abspath(args[i + 1])
        del args[i:i + 2]
    build(verbose=True, extra=args, out=out)
