"""Builds librdkv.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librdkv.so")
# (source, object, extra flags); the mixed-mode decode kernels are compiled once per head-set count and row length
# class so that their many instantiations build in parallel; the slowest objects come first
SOURCES = [
    ("decode_mixed_kernels.hip", "decode_mixed_hs2_long1.o", ["-DRDKV_MIXED_HS=2", "-DRDKV_MIXED_LONG=1"]),
    ("decode_mixed_kernels.hip", "decode_mixed_hs2_long0.o", ["-DRDKV_MIXED_HS=2", "-DRDKV_MIXED_LONG=0"]),
    ("decode_mixed_kernels.hip", "decode_mixed_hs1_long1.o", ["-DRDKV_MIXED_HS=1", "-DRDKV_MIXED_LONG=1"]),
    ("decode_mixed_kernels.hip", "decode_mixed_hs1_long0.o", ["-DRDKV_MIXED_HS=1", "-DRDKV_MIXED_LONG=0"]),
    ("decode_mfma_kernels.hip", "decode_mfma_kernels.o", []),
    ("rdkv_api.hip", "rdkv_api.o", []),
    ("decode_rows_mfma.hip", "decode_rows_mfma.o", []),
    ("decode_kernels.hip", "decode_kernels.o", []),
    ("pack_kernels.hip", "pack_kernels.o", []),
    ("allocate_kernels.hip", "allocate_kernels.o", []),
    ("weights_kernels.hip", "weights_kernels.o", []),
    ("calib_kernels.hip", "calib_kernels.o", []),
]

FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950",
    # packed fp32 instructions are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the quantizer must be reproducible bit for bit: no implicit fused multiply-add
    "-ffp-contract=off",
    # MFMA results stay in ordinary vector registers (no copies through the accumulation registers)
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-function",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def build(verbose=True, jobs=8):
    objs, procs = [], []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src, obj_name, extra in SOURCES:
        obj = os.path.join(HERE, "_build", obj_name)
        objs.append(obj)
        cmd = ["hipcc", "-c", os.path.join(CSRC, src), "-o", obj] + FLAGS + extra
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((obj_name, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        if len(procs) >= jobs:
            _drain(procs)
    _drain(procs)
    cmd = ["hipcc", "-shared", "-o", LIB] + objs + ["--offload-arch=gfx950"]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def _drain(procs):
    while procs:
        src, p = procs.pop(0)
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if out:
            print(out, flush=True)
        if p.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}")


if __name__ == "__main__":
    build()
    print("built", LIB)
