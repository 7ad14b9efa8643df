"""Build the HIP library in-tree: ``python -m paper_2310_19102_amd.build``.

hipcc cross-compiles for gfx950 without a GPU.  Packed-fp32 instruction
selection is switched off for the device pass (the host pass warns that it
does not know the feature; that is harmless), fast-math is never enabled: IEEE
fp32 division and sqrt and unfused multiplies are part of the numerical
contract of the front end.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libatom.so")
SOURCES = ["atom_api.hip", "atom_quantize.hip", "atom_quantize_packed.hip", "atom_gemm.hip", "atom_gemm_big.hip", "atom_gemm_decode.hip", "atom_gemm_gs.hip", "atom_decode_fused.hip", "atom_gemm_f6.hip", "atom_kv.hip", "atom_mx.hip", "atom_calib.hip", "atom_probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-fno-fast-math",
    # MFMA results are consumed by the vector ALU right away: keep them in
    # architectural VGPRs instead of AccVGPRs (saves one copy per element)
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


# per-source overrides: the MX GEMM never touches its accumulators with the vector ALU inside the
# K loop, so its 256 accumulator registers per lane belong in the AccVGPRs; the grouped-query
# attention kernel rescales its accumulators with the vector ALU (online softmax), and with them
# in AccVGPRs every step copied all 32 of them out for a rescaling that rarely runs
SOURCE_FLAGS = {"atom_mx.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=0"],
                "atom_kv.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]}


def build(verbose: bool = False, extra_flags=(), lib: str = LIB, tag: str = "") -> str:
    """Compile every kernel file and link ``libatom.so`` next to this module."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, src.replace(".hip", tag + ".o"))
        cmd = [hipcc, *FLAGS, *SOURCE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    for src, pr in procs:
        out, _ = pr.communicate()
        text = "\n".join(l for l in out.decode().splitlines()
                         if "packed-fp32-ops" not in l and l.strip())
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out.decode()}")
        if verbose and text:
            print(text, flush=True)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
