"""Builds libded_verify.so (HIP, gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import shutil
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libded_verify.so")
SOURCES = ["ded_api.hip", "kernels_shared.hip", "kernels_f32.hip", "kernels_bf16.hip", "gemm_bf16.hip",
           "attn_bf16.hip", "tree_builder.hip", "drafter.hip"]
FLAGS = ["-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
         "-packed-fp32-ops", "-Wall", "-Wno-unused-function"]


def _hipcc() -> str:
    for cand in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = False) -> str:
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    def compile_one(src: str) -> str:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        noise = "not a recognized feature for this target"
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{err}")
        if verbose and err.strip():
            print(err)
        return obj

    with ThreadPoolExecutor(max_workers=6) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    tmp = LIB + ".tmp"
    res = subprocess.run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", tmp],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    os.replace(tmp, LIB)
    return LIB


HOST_ONLY_SOURCES = ["ded_api.hip", "tree_builder.hip", "drafter.hip"]  # validation, sizing, tree builder, draft maker
SAN_LIB = os.path.join(HERE, "_build", "libded_verify_hostsan.so")


def asan_runtime() -> str:
    """The AddressSanitizer runtime of hipcc's clang (to be preloaded into an unsanitized host process)."""
    clang = os.path.join(os.path.dirname(os.path.realpath(_hipcc())), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    res = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = res.stdout.strip()
    if res.returncode != 0 or not os.path.isabs(path) or not os.path.exists(path):
        raise RuntimeError("AddressSanitizer runtime not found")
    return path


def build_host_sanitizer_library() -> str:
    """The same library with AddressSanitizer + UndefinedBehaviorSanitizer in the HOST code of the sources that hold
    the host-side logic (argument validation, workspace sizing, pseudo-sequence builder, draft maker).  Device code is
    never sanitized (every -fsanitize= sits behind -Xarch_host); the kernel objects of the normal build are reused."""
    hipcc = _hipcc()
    objdir = os.path.join(HERE, "_build")
    if not all(os.path.exists(os.path.join(objdir, s.replace(".hip", ".o"))) for s in SOURCES):
        build_library()
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-omit-frame-pointer"]
    flags = ["-O1", "-g"] + [f for f in FLAGS if f != "-O3"]
    objs = []
    for src in SOURCES:
        if src in HOST_ONLY_SOURCES:
            obj = os.path.join(objdir, src.replace(".hip", ".san.o"))
            res = subprocess.run([hipcc, *flags, *san, "-c", os.path.join(CSRC, src), "-o", obj],
                                 capture_output=True, text=True)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc (host sanitizers) failed on {src}:\n{res.stderr}")
        else:
            obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
    res = subprocess.run([hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-Xarch_host", "-fsanitize=address",
                          "-Xarch_host", "-fsanitize=undefined", *objs, "-o", SAN_LIB], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link (host sanitizers) failed:\n" + res.stderr)
    return SAN_LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
