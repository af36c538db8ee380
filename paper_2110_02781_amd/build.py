"""Builds the HIP library in-tree: csrc/*.hip + host sources -> libftp_hip.so (gfx950)."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libftp_hip.so")
OBJ_DIR = os.path.join(HERE, "_build")

COMMON = ["--offload-arch=gfx950", "-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          # MFMA accumulators in ordinary VGPRs: the epilogues read them without accvgpr moves
          "-mllvm", "-amdgpu-mfma-vgpr-form"]
SOURCES = [
    ("k_elem.hip", ["-x", "hip"]),
    ("k_conv.hip", ["-x", "hip"]),
    ("k_gemm.hip", ["-x", "hip"]),
    ("k_fused.hip", ["-x", "hip"]),
    ("k_gemm_deep.hip", ["-x", "hip"]),
    ("stage.cpp", ["-x", "hip"]),
    ("ktrace.cpp", ["-x", "hip"]),
    ("solver.cpp", ["-x", "c++", "-ffp-contract=off"]),
]


def _compile(item):
    src, extra = item
    obj = os.path.join(OBJ_DIR, src + ".o")
    if extra[:2] == ["-x", "c++"]:
        cmd = ["hipcc", "-O2", "-fPIC", "-std=c++17", "-Wall"] + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    else:
        cmd = ["hipcc"] + COMMON + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{out}")
    return src, out


def build(verbose=False):
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=6) as ex:
        for src, out in ex.map(_compile, SOURCES):
            if verbose and out.strip():
                print(f"[{src}]\n{out}")
    objs = [os.path.join(OBJ_DIR, s + ".o") for s, _ in SOURCES]
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
