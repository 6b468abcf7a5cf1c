"""Builds the decode-step HIP library for gfx950, in-tree."""
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libdecodekit.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return [os.path.join(CSRC, "decodekit.hip")]


def _deps():
    out = []
    for root in (CSRC, os.path.join(os.path.dirname(_HERE), "include")):
        for f in os.listdir(root):
            out.append(os.path.join(root, f))
    return out


def up_to_date() -> bool:
    if not os.path.exists(LIB_PATH):
        return False
    t = os.path.getmtime(LIB_PATH)
    return all(os.path.getmtime(f) <= t for f in _deps())


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compiles csrc/ into libdecodekit.so next to this file."""
    if not force and up_to_date():
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    cmd = [hipcc, *HIPCC_FLAGS, *sources(), "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


HOST_SAN_DIR = os.path.join(_HERE, "_build", "host_san")
HOST_SAN_LIB = os.path.join(HOST_SAN_DIR, "libdecodekit_host_san.so")


def build_host_sanitizer_library() -> str:
    """The library's host code under AddressSanitizer and UndefinedBehaviorSanitizer, for tests of
    the host logic on a machine without a GPU (block accounting, prefix index, argument checks):
    the translation unit is compiled for the host only and linked against an EMPTY device bundle,
    so every entry point exists and no kernel does.  The loading process must start with the
    compiler's ASan runtime preloaded (asan_runtime())."""
    os.makedirs(HOST_SAN_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clangxx = os.path.join(_llvm_bin(), "clang++")
    obj, empty, bundle, stub = (os.path.join(HOST_SAN_DIR, n) for n in ("host.o", "empty.hip", "empty.hipfb", "stub.s"))
    subprocess.run([hipcc, "--cuda-host-only", "-c", "-O1", "-g", "-std=c++17", "-fPIC",
                    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
                    "-Wno-unused-function", *sources(), "-o", obj], check=True)
    open(empty, "w").write("\n")
    subprocess.run([hipcc, "--offload-arch=gfx950", "--cuda-device-only", empty, "-o", bundle], check=True)
    # the host object refers to its device bundle by a symbol whose name carries a hash of the unit
    undefined = subprocess.run(["nm", "-u", obj], check=True, capture_output=True, text=True).stdout.split()
    sym = [u for u in undefined if u.startswith("__hip_fatbin_")][0]
    open(stub, "w").write(f'    .section .hip_fatbin,"a",@progbits\n    .globl {sym}\n    .p2align 12\n{sym}:\n'
                          f'    .incbin "{bundle}"\n    .section .note.GNU-stack,"",@progbits\n')
    subprocess.run([clangxx, "-shared", "-fPIC", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", obj, stub,
                    "-o", HOST_SAN_LIB, "-L/opt/rocm/lib", "-lamdhip64"], check=True)
    return HOST_SAN_LIB


def _llvm_bin() -> str:
    return os.environ.get("ROCM_LLVM_BIN", "/opt/rocm/lib/llvm/bin")


def asan_runtime() -> str:
    """Path of the ASan runtime that build_host_sanitizer_library()'s compiler links against."""
    out = subprocess.run([os.path.join(_llvm_bin(), "clang"), "-print-file-name=libclang_rt.asan-x86_64.so"],
                         check=True, capture_output=True, text=True).stdout.strip()
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
