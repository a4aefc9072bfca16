"""Build libdart.so (HIP, gfx950) in-tree: python -m paper_2601_19278_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdart.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
if os.environ.get("DART_TUNING"):          # sweep build: launch tunables become variables
    FLAGS.append("-DDART_TUNING")

# The attention kernel rescales its MFMA accumulators after every key block (running soft-max):
# keep them in ordinary VGPRs, where the multiply needs no copies to and from the accumulation
# registers (the kernel is far from the register limit).
PER_FILE = {"k_attn_mfma.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def build(verbose: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)

    def compile_one(name: str) -> str:
        obj = os.path.join(OBJ, name[:-4] + ".o")
        cmd = [HIPCC, *FLAGS, *PER_FILE.get(name, []), "-c", os.path.join(CSRC, name), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"
        err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}:\n{err}")
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, sources()))
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB],
                         capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n" + res.stderr)
    if verbose:
        print("built", LIB)
    return LIB


SAN_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
             "-Xarch_host", "-fno-omit-frame-pointer", "-Xarch_host", "-fno-sanitize-recover=undefined",
             "-g"]


def build_sanitized(verbose: bool = True, jobs: int = 8) -> str:
    """Host-side AddressSanitizer + UndefinedBehaviorSanitizer build of the whole library, linked
    with tests/abi_host_check.cpp into _build/abi_host_check_san (device code is compiled as
    usual; GPU sanitizers are not used).  The program exercises the ABI's argument checks and
    error paths on the host; it needs no GPU."""
    san = os.path.join(OBJ, "san")
    os.makedirs(san, exist_ok=True)
    check = os.path.join(os.path.dirname(HERE), "tests", "abi_host_check.cpp")

    def compile_one(src: str) -> str:
        obj = os.path.join(san, os.path.basename(src).rsplit(".", 1)[0] + ".o")
        lang = ["-x", "hip"] if src.endswith(".cpp") else []
        cmd = [HIPCC, *FLAGS, *SAN_FLAGS, *PER_FILE.get(os.path.basename(src), []), *lang, "-c", src, "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc (sanitized) failed on {src}:\n{res.stderr}")
        return obj

    srcs = [os.path.join(CSRC, f) for f in sources()] + [check]
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, srcs))
    exe = os.path.join(OBJ, "abi_host_check_san")
    res = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined",
                          *objs, "-o", exe], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link (sanitized) failed:\n" + res.stderr)
    if verbose:
        print("built", exe)
    return exe


if __name__ == "__main__":
    if "--sanitize" in sys.argv[1:]:
        build_sanitized()
    else:
        build()
