"""Builds libptq4vm.so (HIP kernels + C ABI) for gfx950, in-tree next to this file."""
from __future__ import annotations

import concurrent.futures
import glob
import hashlib
import os
import shutil
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libptq4vm.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    # IEEE fp32 division (the quantizer's reciprocal steps must be correctly rounded)
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-fno-fast-math",
    # never let the compiler form packed-fp32 VALU instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall",
    "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")) + glob.glob(os.path.join(CSRC, "*.cpp")))


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", shutil.which("hipcc")):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


OBJ_DIR = os.path.join(_HERE, "_build")


def _headers():
    return sorted(glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(_HERE, "..", "include", "*.h")))


# Host code only: on a hipcc line each -fsanitize= goes directly after -Xarch_host (GPU sanitizers are not available).
SANITIZE_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-fno-omit-frame-pointer", "-g"]
SANITIZED_LIB_PATH = os.path.join(_HERE, "libptq4vm_asan.so")


def _compile_one(src: str, force: bool, extra=()):
    """Compile one source to an object file; returns (object path, compiler log)."""
    h = hashlib.sha1()
    for path in [src, *_headers()]:
        with open(path, "rb") as f:
            h.update(f.read())
    h.update(" ".join([*HIPCC_FLAGS, *extra]).encode())
    obj = os.path.join(OBJ_DIR, os.path.basename(src) + "." + h.hexdigest()[:16] + ".o")
    if not force and os.path.exists(obj):
        return obj, ""
    flags = [f for f in HIPCC_FLAGS if f != "-shared"] + list(extra)
    tmp = obj + f".tmp{os.getpid()}"
    res = subprocess.run([hipcc(), *flags, "-x", "hip", "-c", src, "-o", tmp], capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n" + res.stdout + res.stderr)
    os.replace(tmp, obj)
    return obj, res.stdout + res.stderr


def build(verbose: bool = False, force: bool = True) -> str:
    """Compile every source under csrc/ (one hipcc process per file, in parallel) and link
    libptq4vm.so.  force=True recompiles everything; force=False reuses an object file whose source,
    headers and flags are unchanged (a convenience while iterating on one kernel)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        results = list(pool.map(lambda s: _compile_one(s, force), srcs))
    keep = {obj for obj, _ in results}
    for stale in glob.glob(os.path.join(OBJ_DIR, "*.o")):
        if stale not in keep:
            os.remove(stale)
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    link = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *sorted(keep), "-o", tmp],
                          capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    log = "\n".join(l for _, out in results for l in out.splitlines() if noise not in l)
    log += "\n".join(l for l in (link.stdout + link.stderr).splitlines() if noise not in l)
    if link.returncode != 0:
        raise RuntimeError("link failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def build_sanitized() -> str:
    """libptq4vm_asan.so: the same sources with AddressSanitizer and UndefinedBehaviorSanitizer on the HOST half
    (argument checks, launch set-up, status strings); the device code is compiled as always.  Load it with
    PTQ4VM_LIB=<path> and clang's ASan runtime preloaded (see tests/test_sanitized_host.py)."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    srcs = sources()
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, len(srcs))) as pool:
        results = list(pool.map(lambda s: _compile_one(s, False, SANITIZE_FLAGS), srcs))
    objs = sorted(obj for obj, _ in results)
    link = subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-shared-libsan", "-fsanitize=address",
                           "-fsanitize=undefined", *objs, "-o", SANITIZED_LIB_PATH], capture_output=True, text=True)
    if link.returncode != 0:
        raise RuntimeError("link failed:\n" + link.stdout + link.stderr)
    return SANITIZED_LIB_PATH


def sanitizer_runtime() -> str:
    """Path of clang's shared ASan runtime (to preload into the Python process that loads the sanitized library)."""
    res = subprocess.run([hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True, check=True)
    return res.stdout.strip()


if __name__ == "__main__":
    import sys

    if "--sanitize" in sys.argv:
        print(build_sanitized())
    else:
        print(build(verbose=True, force="--incremental" not in sys.argv))
