"""Builds libptenc.so (hand-written gfx950 HIP kernels + the C-ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libptenc.so")
SOURCES = ["ptenc_api.hip", "cache_kernels.hip", "attn_generic.hip", "decode_mfma.hip", "util_kernels.hip", "adapter_kernels.hip",
           "stack_api.hip", "scored_kernels.hip"]
# packed-fp32 instruction selection is switched off for all device code
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]
# The step kernel's leading scalar arguments (list and mask pointers, counter pointers, the cache
# pointer, two sizes: the 14 dwords that fit) are preloaded into SGPRs at wavefront launch, so its
# first loads need not wait for the argument block; the compiler keeps a prologue that loads them the
# ordinary way where the firmware does not preload.
EXTRA_FLAGS = {"decode_mfma.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=16"]}
OBJ_DIR = os.path.join(PKG_DIR, "_build")


def hipcc_path() -> str:
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc"):
        if p and os.path.exists(p):
            return p
    return "hipcc"


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only feature flag and says so once per source
    out = "\n".join(l for l in res.stdout.splitlines() if "not a recognized feature" not in l)
    if res.returncode != 0:
        raise RuntimeError("%s failed:\n%s" % (os.path.basename(cmd[0]), out))
    if verbose and out.strip():
        print(out)


def build(verbose: bool = True) -> str:
    """Compiles every HIP source for gfx950 (one object each, in parallel) and links one shared library; returns its path."""
    from concurrent.futures import ThreadPoolExecutor
    os.makedirs(OBJ_DIR, exist_ok=True)
    objs = [os.path.join(OBJ_DIR, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc_path()] + HIPCC_FLAGS + EXTRA_FLAGS.get(s, []) + ["-c", os.path.join(CSRC, s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH + ".tmp"], verbose)
    os.replace(LIB_PATH + ".tmp", LIB_PATH)
    build_c_smoke(verbose)
    return LIB_PATH


SAN_LIB_PATH = os.path.join(OBJ_DIR, "libptenc_hostsan.so")
SAN_SOURCES = ("ptenc_api.hip", "stack_api.hip")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-g"]


def sanitizer_runtime() -> str:
    """The AddressSanitizer runtime of the compiler that builds the library (to be preloaded into a host
    program that was not built with it, such as the Python interpreter)."""
    res = subprocess.run([hipcc_path().replace("hipcc", "amdclang++"), "-print-file-name=libclang_rt.asan-x86_64.so"],
                         stdout=subprocess.PIPE, text=True)
    path = res.stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        raise RuntimeError("AddressSanitizer runtime not found")
    return os.path.realpath(path)


def build_host_sanitized(verbose: bool = False) -> str:
    """The same library with its HOST code (argument checks, context bookkeeping, launch glue) built with
    AddressSanitizer and UndefinedBehaviorSanitizer; device code is built as always.  For host-only tests:
    it is kept beside the objects, never next to the real library, and nothing loads it by default
    (PTENC_LIB selects it)."""
    from concurrent.futures import ThreadPoolExecutor
    san_dir = os.path.join(OBJ_DIR, "hostsan")
    os.makedirs(san_dir, exist_ok=True)
    # the host glue is in these two sources; the others hold kernels and their one-line launchers, and their
    # objects are taken from the ordinary build
    objs, cmds = [], []
    for s in SOURCES:
        if s in SAN_SOURCES:
            o = os.path.join(san_dir, s.replace(".hip", ".o"))
            cmds.append([hipcc_path()] + HIPCC_FLAGS + SAN_FLAGS + EXTRA_FLAGS.get(s, []) + ["-c", os.path.join(CSRC, s), "-o", o])
        else:
            o = os.path.join(OBJ_DIR, s.replace(".hip", ".o"))
            if not os.path.exists(o):
                raise RuntimeError("%s is missing: run build() first" % o)
        objs.append(o)
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", "-Xarch_host", "-fsanitize=address",
          "-Xarch_host", "-fsanitize=undefined", "-shared-libsan"] + objs + ["-o", SAN_LIB_PATH + ".tmp"], verbose)
    os.replace(SAN_LIB_PATH + ".tmp", SAN_LIB_PATH)
    return SAN_LIB_PATH


TIMELINE_LIB_PATH = os.path.join(PKG_DIR, "libptenc_timeline.so")


def build_timeline(verbose: bool = False) -> str:
    """The same library with -DPTENC_TIMELINE: the step kernel notes the wall clock at the boundaries of its phases
    (entry, walk begins, walk ends, wavefronts merged, result out, ...) per workgroup, at the end of the state block.
    A profiling build for `python -m paper_2602_16839_amd.step_timeline`, which selects it through PTENC_LIB; nothing
    else loads it."""
    from concurrent.futures import ThreadPoolExecutor
    tl_dir = os.path.join(OBJ_DIR, "timeline")
    os.makedirs(tl_dir, exist_ok=True)
    objs = [os.path.join(tl_dir, s.replace(".hip", ".o")) for s in SOURCES]
    cmds = [[hipcc_path()] + HIPCC_FLAGS + ["-DPTENC_TIMELINE"] + EXTRA_FLAGS.get(s, []) + ["-c", os.path.join(CSRC, s), "-o", o]
            for s, o in zip(SOURCES, objs)]
    with ThreadPoolExecutor(max_workers=min(8, len(cmds))) as pool:
        list(pool.map(lambda c: _run(c, verbose), cmds))
    _run([hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", TIMELINE_LIB_PATH + ".tmp"], verbose)
    os.replace(TIMELINE_LIB_PATH + ".tmp", TIMELINE_LIB_PATH)
    return TIMELINE_LIB_PATH


C_SMOKE_SRC = os.path.join(ROOT, "tests", "c_abi", "abi_smoke.c")
C_SMOKE_BIN = os.path.join(ROOT, "tests", "c_abi", "abi_smoke")


def build_c_smoke(verbose: bool = True) -> str:
    """A plain C program (gcc, no HIP compiler) that drives the library through include/ptenc.h."""
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I" + os.path.join(ROOT, "include"),
           "-I" + os.path.join(rocm, "include"), C_SMOKE_SRC, "-o", C_SMOKE_BIN + ".tmp",
           "-L" + PKG_DIR, "-lptenc", "-Wl,-rpath,$ORIGIN/../../paper_2602_16839_amd",
           "-L" + os.path.join(rocm, "lib"), "-lamdhip64", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-lm"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("gcc failed:\n" + res.stdout)
    os.replace(C_SMOKE_BIN + ".tmp", C_SMOKE_BIN)
    return C_SMOKE_BIN


if __name__ == "__main__":
    build()
    if "--timeline" in sys.argv[1:]:
        print(build_timeline(verbose=True))
    sys.exit(0)
