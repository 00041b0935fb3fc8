"""Build libfsf.so (HIP kernels + C ABI + host composer) for gfx950 with hipcc.

Usage:  python -m paper_2401_08671_amd.build               # the library, next to this file
        python -m paper_2401_08671_amd.build --sanitize    # also the sanitized host-code build
The library is written next to this file so it travels with the source tree.

--sanitize builds a second copy of the library whose HOST code (composer, allocator, the
attention call's planning and validation) is compiled with AddressSanitizer and
UndefinedBehaviorSanitizer (device code as usual), and tests/native/host_check.cpp against it:
_build/asan/libfsf_asan.so and _build/asan/host_check, which tests/test_sanitized_host.py runs
on the CPU.
"""
from __future__ import annotations

import concurrent.futures
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.environ.get("FSF_LIB_PATH", os.path.join(HERE, "libfsf.so"))

# -packed-fp32-ops is switched off on purpose: packed fp32 forms have given wrong results on the test machines.
HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wno-unused-command-line-argument", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith((".hip", ".cpp")))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    cmd = ["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + HIP_FLAGS
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    warn = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l and l.strip())
    if warn:
        sys.stderr.write(warn + "\n")
    return obj


def build(verbose: bool = True) -> str:
    if shutil.which("hipcc") is None:
        raise RuntimeError("hipcc not found on PATH")
    os.makedirs(OBJ_DIR, exist_ok=True)
    # the prefill tile's instruction sequence is a generated header
    r = subprocess.run([sys.executable, os.path.join(CSRC, "gen_prefill_sequence.py")], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gen_prefill_sequence.py failed:\n{r.stdout}\n{r.stderr}")
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    tmp = LIB_PATH + ".tmp"
    cmd = ["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    os.replace(tmp, LIB_PATH)
    if verbose:
        print(f"built {LIB_PATH} from {len(srcs)} sources")
    return LIB_PATH


SAN_DIR = os.path.join(OBJ_DIR, "asan")
SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
HOST_CHECK = os.path.join(SAN_DIR, "host_check")


def _compile_sanitized(src: str) -> str:
    obj = os.path.join(SAN_DIR, os.path.splitext(src)[0] + ".o")
    flags = [f for f in HIP_FLAGS if f != "-O3"] + ["-O1"] + SAN_FLAGS
    r = subprocess.run(["hipcc", "-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj] + flags, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc (sanitized) failed on {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build_sanitized(verbose: bool = True) -> str:
    """libfsf_asan.so (host code under ASan + UBSan) and the host_check program that drives it."""
    if shutil.which("hipcc") is None:
        raise RuntimeError("hipcc not found on PATH")
    os.makedirs(SAN_DIR, exist_ok=True)
    r = subprocess.run([sys.executable, os.path.join(CSRC, "gen_prefill_sequence.py")], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gen_prefill_sequence.py failed:\n{r.stdout}\n{r.stderr}")
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile_sanitized, srcs))
    lib = os.path.join(SAN_DIR, "libfsf_asan.so")
    san_link = ["-fsanitize=address", "-fsanitize=undefined"]
    r = subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + san_link + objs,
                       capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link (sanitized) failed:\n{r.stdout}\n{r.stderr}")
    clangxx = os.path.join(os.path.dirname(os.path.realpath(shutil.which("hipcc"))), "..", "lib", "llvm", "bin", "clang++")
    if not os.path.exists(clangxx):
        clangxx = "/opt/rocm/lib/llvm/bin/clang++"
    cmd = [clangxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fno-sanitize-recover=undefined"] + san_link + [
        "-I" + os.path.join(ROOT, "include"), os.path.join(ROOT, "tests", "native", "host_check.cpp"),
        "-L" + SAN_DIR, "-lfsf_asan", "-Wl,-rpath," + SAN_DIR, "-o", HOST_CHECK]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"host_check build failed:\n{r.stdout}\n{r.stderr}")
    if verbose:
        print(f"built {lib} and {HOST_CHECK}")
    return HOST_CHECK


if __name__ == "__main__":
    build()
    if "--sanitize" in sys.argv[1:]:
        build_sanitized()
