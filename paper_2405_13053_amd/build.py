"""Builds libmeteora.so (gfx950) in-tree with hipcc.  Run on the CPU host; no GPU needed."""
from __future__ import annotations

import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libmeteora.so")
# measurement tools, see csrc/diag/*.hip
DIAG_TOOLS = ("mfma_ceiling", "operand_path_probe")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def _hipcc(cmd, verbose):
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    """Compile every HIP source into one shared library, and the stand-alone measurement tools
    (csrc/diag/<tool>.hip -> ./<tool>); always recompiles."""
    tmp = LIB + f".tmp{os.getpid()}"
    _hipcc(["hipcc", *HIPCC_FLAGS, "-o", tmp, *sources()], verbose)
    os.replace(tmp, LIB)
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    for tool in DIAG_TOOLS:
        exe = os.path.join(HERE, tool)
        tmp = exe + f".tmp{os.getpid()}"
        _hipcc(["hipcc", *flags, "-o", tmp, os.path.join(HERE, "csrc", "diag", tool + ".hip")], verbose)
        os.replace(tmp, exe)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
