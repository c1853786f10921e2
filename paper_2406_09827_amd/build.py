"""Builds libhipattn.so (the C-ABI GPU library) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhipattn.so")
CSRC_AUX = os.path.join(HERE, "csrc_aux")
LIB_AUX = os.path.join(HERE, "libhipattn_aux.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
# -fno-honor-nans: max/min compile to single instructions (no NaN quieting); infinities are
# still honoured (the kernels use -inf as "no score").  NaN inputs are outside the contract.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-fno-honor-nans",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    """Kernel sources, the translation units with the most template instantiations first (they take the
    longest, so starting them first shortens the parallel build)."""
    heavy = ("mask_decode", "mask_mfma_bk", "attn_decode", "attn_mfma")
    names = sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))
    return sorted(names, key=lambda n: next((i for i, h in enumerate(heavy) if n.startswith(h)), len(heavy)))


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, src[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    return obj


def build_lib(jobs: int = 8) -> str:
    """Compile every kernel source and link the shared library (always rebuilds)."""
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(_compile, sources()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")
    return LIB


def build_aux() -> str:
    """The test and measurement aids (include/hipattn_aux.h): a library of their own, so that the product
    library exports the method's calls only."""
    cmd = [HIPCC, *FLAGS, "-shared", os.path.join(CSRC_AUX, "probes.hip"), "-o", LIB_AUX]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on probes.hip:\n{r.stdout}\n{r.stderr}")
    return LIB_AUX


def build_c_example() -> str:
    """Compile the plain-C caller of the ABI (tests/c_abi/c_abi_smoke.c) with gcc against the built
    library; the GPU tests run the binary.  Also proves that include/hipattn.h is valid C."""
    root = os.path.dirname(HERE)
    src = os.path.join(root, "tests", "c_abi", "c_abi_smoke.c")
    exe = os.path.join(root, "tests", "c_abi", "c_abi_smoke")
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(HIPCC)))
    cmd = ["gcc", "-std=c11", "-Wall", "-O1", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(root, "include"),
           "-I", os.path.join(rocm, "include"), src, "-o", exe, "-L", HERE, "-lhipattn",
           "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../../paper_2406_09827_amd", "-Wl,-rpath," + os.path.join(rocm, "lib")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"gcc failed on {src}:\n{r.stdout}\n{r.stderr}")
    return exe


if __name__ == "__main__":
    print(build_lib())
    print(build_aux())
    print(build_c_example())
