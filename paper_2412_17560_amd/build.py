"""Build libgqsa.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
# the library the binding loads: the in-tree build, unless GQSA_LIBRARY names another one (the
# sanitizer leg of the tests points it at the host-only build below)
LIB = os.environ.get("GQSA_LIBRARY") or os.path.join(HERE, "libgqsa.so")
HOST_ONLY = bool(os.environ.get("GQSA_LIBRARY"))
SANITIZED_LIB = os.path.join(OBJ, "libgqsa_host_asan.so")

# (gqsa_gemv.hip is compiled four times: whole, and once per further tile size -- "file:part")
SOURCES = ["gqsa_gemv.hip", "gqsa_gemv.hip:1", "gqsa_gemv.hip:2", "gqsa_gemv.hip:3", "gqsa_gemv.hip:4", "gqsa_pack.cpp",
           "gqsa_panels.cpp", "gqsa_api.cpp", "gqsa_panel_kernel.hip", "gqsa_pack_device.hip", "gqsa_baselines.hip"]

COMMON = ["-O3", "-fPIC", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
          "-Wall", "-Wextra", "-Wno-unused-parameter"]
# device code: gfx950 only; packed-fp32 instruction selection is switched off
HIP_FLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-ffp-contract=off"]   # fused multiply-adds only where the source asks for them
# the GEMV kernel's ten leading scalar parameters arrive in scalar registers at wavefront start
# (kernel-argument preloading) instead of being loaded from the argument block first
EXTRA_HIP_FLAGS = {"gqsa_gemv.hip": ["-mllvm", "-amdgpu-kernarg-preload-count=14"]}
# host arithmetic of the quantiser: every fp32 operation is a single IEEE operation
HOST_FLAGS = ["-ffp-contract=off", "-fno-fast-math"]


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _compile(src: str) -> str:
    src, _, part = src.partition(":")
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + (f"_part{part}" if part else "") + ".o")
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        defines = [f"-DGQSA_GEMV_PART={part}"] if part else []
        cmd = [_hipcc(), *COMMON, *HIP_FLAGS, *EXTRA_HIP_FLAGS.get(os.path.basename(path), []), *defines, "-c", path, "-o", obj]
    else:
        cmd = [_hipcc(), *COMMON, *HOST_FLAGS, "-x", "c++", "-c", path, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"compile failed: {' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    noise = "is not a recognized feature for this target"
    warn = "\n".join(l for l in r.stderr.splitlines() if noise not in l).strip()
    if warn:
        print(warn)
    return obj


def build() -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(_compile, SOURCES))
    cmd = [_hipcc(), "-shared", "-fPIC", "--offload-arch=gfx950", *objs, "-o", LIB, "-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed: {' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    return LIB


def build_sanitized() -> str:
    """Host-only build of the library -- packer, image builders and the C boundary, the device
    side replaced by stubs that answer GQSA_ERR_HIP -- with AddressSanitizer and
    UndefinedBehaviorSanitizer (host code only; no GPU code is compiled or sanitized)."""
    os.makedirs(OBJ, exist_ok=True)
    srcs = [os.path.join(CSRC, f) for f in ("gqsa_pack.cpp", "gqsa_panels.cpp", "gqsa_api.cpp", "gqsa_host_stubs.cpp")]
    cmd = [_hipcc(), "-x", "c++", "-O1", "-g", "-fPIC", "-shared", "-std=c++17", "-fno-gpu-sanitize",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-shared-libsan", "-fno-omit-frame-pointer",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC, *HOST_FLAGS, *srcs, "-o", SANITIZED_LIB, "-lpthread"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"sanitizer build failed: {' '.join(cmd)}\n{r.stdout}\n{r.stderr}")
    return SANITIZED_LIB


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime the sanitized library needs preloaded."""
    r = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = r.stdout.strip()
    if os.path.isabs(path) and os.path.exists(path):
        return path
    r = subprocess.run([_hipcc(), "--print-runtime-dir"], capture_output=True, text=True)
    return os.path.join(r.stdout.strip(), "libclang_rt.asan-x86_64.so")


if __name__ == "__main__":
    import sys
    print(build_sanitized() if "--asan" in sys.argv[1:] else build())
