"""Builds libclear_attn.so (gfx950) in-tree with hipcc.  Run: python -m paper_2412_16112_amd.build"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libclear_attn.so")
SOURCES = ["clear_attn_api.cpp", "schedule.cpp", "kernels_bf16.hip", "kernels_bf16_d64.hip", "kernels_f32.hip", "mfma_peak.hip", "band_merge.hip", "kernels_bf16_bwd.hip", "kernels_bf16_bwd_d64.hip", "prologue.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",  # no packed-fp32 instructions
    "-Wno-unused-command-line-argument", "-Wno-unknown-attributes",
]


def build(verbose=False, extra_flags=()):
    """Compile every source for gfx950 and link the shared library.  Always recompiles."""
    cmd = ["hipcc", *FLAGS, *extra_flags, "-x", "hip"]
    cmd += [os.path.join(CSRC, s) for s in SOURCES]
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd += ["-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, extra_flags=sys.argv[1:]))
