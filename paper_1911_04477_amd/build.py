"""Build libbnn.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libbnn.so")
OBJ_DIR = os.path.join(HERE, "_build")
SOURCES = ["api.hip", "encode.hip", "im2col.hip", "gemm.hip", "gemm_lowk.hip", "gemm_latency.hip", "conv.hip", "glue.hip", "mfma.hip", "control.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed-FP32 VALU forms are disabled for all device code of this library.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-Wall", "-Wno-unused-function",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]

# conv.hip: the matrix-core first layer reads its accumulators on the vector unit; keeping them in
# ordinary vector registers (not accumulation registers) saves a move per element, and those
# moves queue behind the matrix instruction in flight.
EXTRA_FLAGS = {"conv.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


# Checker build of the HOST side (argument validation, dispatch, launch code) with AddressSanitizer
# and UndefinedBehaviorSanitizer; device code is compiled as usual.  CPU-only use:
#   python paper_1911_04477_amd/build.py --sanitize
#   LD_PRELOAD="$(gcc -print-file-name=libasan.so) $(gcc -print-file-name=libubsan.so)" ASAN_OPTIONS=detect_leaks=0 \
#       BNN_SANITIZE=1 python -m pytest tests/test_abi_host.py
SAN_LIB = os.path.join(HERE, "libbnn_san.so")
SAN_HOST_FLAGS = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                  "-fno-omit-frame-pointer", "-g"]


def build_sanitized() -> str:
    out_dir = os.path.join(OBJ_DIR, "san")
    os.makedirs(out_dir, exist_ok=True)
    flags = [f if f != "-O3" else "-O1" for f in FLAGS]

    def comp(src: str) -> str:
        obj = os.path.join(out_dir, os.path.splitext(src)[0] + ".o")
        subprocess.check_call([HIPCC, *flags, *SAN_HOST_FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src),
                               "-o", obj])
        return obj

    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(comp, SOURCES))
    tmp = SAN_LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-Xarch_host", "-fsanitize=address",
                           "-Xarch_host", "-fsanitize=undefined", *objs, "-o", tmp])
    os.replace(tmp, SAN_LIB)
    return SAN_LIB


def _compile(src: str) -> str:
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    subprocess.check_call([HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), "-c", os.path.join(CSRC, src), "-o", obj])
    return obj


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", tmp])
    os.replace(tmp, LIB)
    if verbose:
        print("built", LIB)
    return LIB


if __name__ == "__main__":
    import sys
    if "--sanitize" in sys.argv[1:]:
        print("built", build_sanitized())
    else:
        build(verbose=True)
