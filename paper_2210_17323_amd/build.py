"""Builds libgptq_mi355.so from csrc/*.hip with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libgptq_mi355.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-DNDEBUG",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument",
         "-Wno-ignored-optimization-argument"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{p.stderr}")
    return obj


def build(verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    p = subprocess.run(cmd, capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError(f"link failed:\n{p.stderr}")
    if verbose:
        print(f"built {LIB} from {len(srcs)} sources", file=sys.stderr)
    return LIB


SAN_DIR = os.path.join(OBJ, "host_sanitize")
SAN_BIN = os.path.join(SAN_DIR, "host_check")
SAN_MAIN = os.path.join(os.path.dirname(HERE), "tests", "host_sanitize_main.cpp")
SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def _compile_sanitized(src: str) -> str:
    obj = os.path.join(SAN_DIR, src[:-4] + ".o")
    flags = [f for f in FLAGS if f not in ("-O3", "-fvisibility=hidden")] + ["-O1", "-g", "-w", *SAN_HOST]
    p = subprocess.run([HIPCC, *flags, "-c", os.path.join(CSRC, src), "-o", obj], capture_output=True, text=True)
    if p.returncode != 0:
        raise RuntimeError(f"hipcc (host sanitizers) failed on {src}:\n{p.stderr}")
    return obj


def build_host_sanitized(verbose: bool = True) -> str:
    """The library's sources with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST code only (device code as
    usual; there is no GPU sanitizer here), linked with tests/host_sanitize_main.cpp into an executable that walks
    every entry point's validation and workspace arithmetic.  Takes a few minutes; returns the executable's path."""
    os.makedirs(SAN_DIR, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile_sanitized, srcs))
    main_o = os.path.join(SAN_DIR, "main.o")
    clang = os.path.join(os.path.dirname(HIPCC), "..", "lib", "llvm", "bin", "clang++")
    for cmd in ([clang, "-O1", "-g", "-std=c++17", "-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer", "-c", SAN_MAIN, "-o", main_o],
                [HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", main_o, *objs, "-o", SAN_BIN]):
        p = subprocess.run(cmd, capture_output=True, text=True)
        if p.returncode != 0:
            raise RuntimeError(f"{' '.join(cmd[:2])} ... failed:\n{p.stderr}")
    if verbose:
        print(f"built {SAN_BIN}", file=sys.stderr)
    return SAN_BIN


def host_sanitized_is_current() -> bool:
    if not os.path.exists(SAN_BIN):
        return False
    built = os.path.getmtime(SAN_BIN)
    deps = [os.path.join(CSRC, f) for f in os.listdir(CSRC)] + [SAN_MAIN, os.path.join(os.path.dirname(HERE), "include", "gptq.h")]
    return all(os.path.getmtime(d) <= built for d in deps)


if __name__ == "__main__":
    if "--host-sanitize" in sys.argv[1:]:
        sys.exit(subprocess.run([build_host_sanitized()]).returncode)
    build()
