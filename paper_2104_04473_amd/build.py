"""Builds libptdp.so (the C-ABI library) in-tree with hipcc for gfx950.

Usage: python -m paper_2104_04473_amd.build [--sanitize]

--sanitize builds libptdp_asan.so instead: the same sources with AddressSanitizer and UndefinedBehaviorSanitizer
on the host pass only (argument checks, stash / workspace layout, schedule builder, GEMM planning), device code
unchanged.  Load it with PTDP_LIB=<path> and the sanitizer runtime preloaded (see tests/test_host_sanitized.py).
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libptdp.so")
SOURCES = ["api.hip", "elementwise.hip", "gemm.hip", "attention.hip", "lm_stage.hip", "ceilings.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# per-source additions.  attention.hip: one wave per SIMD, so every instruction counts; with MFMA results in the
# vector registers (instead of the accumulation registers) the softmax arithmetic reads them in place and the main
# loops lose a quarter of their instructions (v_accvgpr moves).
EXTRA_FLAGS = {"attention.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}

LIB_ASAN = os.path.join(HERE, "libptdp_asan.so")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-omit-frame-pointer", "-g"]


def _compile(src, sanitize=False):
    obj = os.path.join(HERE, "_build", ("asan_" if sanitize else "") + src.replace(".hip", ".o"))
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + SAN_FLAGS if sanitize else FLAGS
    cmd = [HIPCC] + flags + EXTRA_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s\n%s" % (src, r.stdout, r.stderr))
    return obj


def sanitizer_runtime():
    """Path of the AddressSanitizer runtime that a process loading libptdp_asan.so must preload."""
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "lib", "llvm", "bin", "clang")
    r = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    return r.stdout.strip()


def build(verbose=True, sanitize=False):
    """Compiles every HIP source and links libptdp.so (always recompiles); sanitize=True: libptdp_asan.so."""
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(lambda src: _compile(src, sanitize), SOURCES))
    lib = LIB_ASAN if sanitize else LIB
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + objs
    if sanitize:
        cmd += ["-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n%s\n%s" % (r.stdout, r.stderr))
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build(sanitize="--sanitize" in sys.argv[1:])
    sys.exit(0)
