"""Build libpdelta.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2512_19720_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
OBJ = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libpdelta.so")

SOURCES = ["pdelta_api.hip", "pdelta_pack.hip", "pdelta_pack_group.hip", "pdelta_patch.hip", "pdelta_linear_skinny.hip",
           "pdelta_linear_gemm.hip", "pdelta_linear_variants.hip", "pdelta_grad.hip", "pdelta_probes.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",     # no packed-fp32 codegen
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _compile(src: str, obj_dir: str = OBJ, extra=()) -> str:
    obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
    env_extra = os.environ.get("PDELTA_EXTRA_HIPCC_FLAGS", "").split()   # developer builds (e.g. -D switches)
    cmd = [_hipcc(), *HIPCC_FLAGS, *env_extra, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = ("is not a recognized feature for this target",         # host pass ignores the GPU feature
             "option as it is not currently supported for target 'amdgcn")   # host-only sanitizer flags
    err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip() and not extra:
        sys.stderr.write(err + "\n")
    return obj


def build_library(jobs: int = 5, lib_path: str = LIB, obj_dir: str = OBJ, extra_compile=(), extra_link=()) -> str:
    """Compile every source for gfx950 and link the shared library (libpdelta.so in-tree unless
    another path is given).  Always recompiles."""
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda src: _compile(src, obj_dir, tuple(extra_compile)), SOURCES))
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *extra_link, "-o", lib_path, *objs]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"link failed:\n{res.stderr}")
    return lib_path


# Host-side sanitizers: AddressSanitizer and UndefinedBehaviorSanitizer on the host pass only
# (the device code is compiled as usual); used by tests/test_sanitizers.py.
SANITIZE_COMPILE = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
                    "-Xarch_host", "-fno-sanitize-recover=undefined"]
SANITIZE_LINK = ["-fsanitize=address", "-fsanitize=undefined", "-shared-libasan"]


def sanitizer_runtime() -> str:
    """Path of clang's shared AddressSanitizer runtime (to be preloaded into an uninstrumented python)."""
    out = subprocess.run([_hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True)
    path = out.stdout.strip()
    if not os.path.isabs(path):
        import glob
        hits = glob.glob("/opt/rocm/lib/llvm/lib/clang/*/lib/linux/libclang_rt.asan-x86_64.so")
        path = hits[0] if hits else ""
    return path


if __name__ == "__main__":
    print(build_library())
