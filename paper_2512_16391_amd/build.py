"""Builds libkascade.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libkascade.so")

SOURCES = ["api.hip", "decode_kernels.hip", "decode_mfma_kernels.hip", "topk_kernels.hip", "prefill_kernels.hip", "calib_kernels.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-ffp-contract=fast",
    # keep MFMA accumulators in VGPRs: the softmax reads them right away, AGPR copies cost VALU slots
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    # the sources compile side by side
    "-parallel-jobs=6",
]


def hipcc_path():
    return shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


def build_library(verbose=True, extra_flags=()):
    srcs = [os.path.join(CSRC, s) for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    cmd = [hipcc_path(), *HIPCC_FLAGS, *extra_flags, *srcs, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless
    err = "\n".join(ln for ln in res.stderr.splitlines() if "packed-fp32-ops" not in ln)
    if res.returncode != 0:
        sys.stderr.write(res.stderr)
        raise RuntimeError("hipcc failed building libkascade.so")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    return LIB_PATH


if __name__ == "__main__":
    build_library()
