"""Build libtreetrain.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtreetrain.so")

SOURCES = ["tt_error.cpp", "tt_meta.cpp", "tt_api.hip", "tt_timing.hip", "tt_attn_ref.hip", "tt_loss.hip",
           "tt_attn_fwd.hip", "tt_attn_bwd.hip", "tt_attn_dkdv.hip", "tt_rope.hip", "tt_partition.cpp",
           "tt_partition_run.hip", "tt_conv.hip", "tt_gdn.hip", "tt_gdn_bwd.hip"]

# Kernels that run two waves per SIMD keep MFMA results in architectural VGPRs (the softmax / dS
# arithmetic consumes them directly); the dK/dV kernel needs the accumulation VGPRs for its 128
# accumulator registers per lane and is compiled with the default register form.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
PER_FILE_FLAGS = {"tt_attn_fwd.hip": VGPR_FORM, "tt_attn_bwd.hip": VGPR_FORM, "tt_gdn.hip": VGPR_FORM}

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
    "-Wno-unused-parameter",
    # packed-fp32 code generation is switched off for every HIP translation unit
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every source (always; no staleness check) and link the shared library."""
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    srcs = [s for s in SOURCES if os.path.exists(os.path.join(CSRC, s))]
    missing = [s for s in SOURCES if s not in srcs]
    if missing:
        raise RuntimeError(f"missing sources: {missing}")
    procs = []
    objs = []
    for s in srcs:
        obj = os.path.join(objdir, os.path.splitext(s)[0] + ".o")
        objs.append(obj)
        lang = ["-x", "hip"] if s.endswith(".hip") else []
        cmd = [hipcc()] + HIPCC_FLAGS + PER_FILE_FLAGS.get(s, []) + list(extra_flags) + lang + ["-c", os.path.join(CSRC, s), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((s, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for s, p in procs:
        out, _ = p.communicate()
        lines = [ln for ln in out.splitlines() if "packed-fp32-ops" not in ln and ln.strip()]
        if p.returncode != 0:
            failed = True
            print(f"--- {s} FAILED\n{out}", file=sys.stderr)
        elif verbose and lines:
            print(f"--- {s}\n" + "\n".join(lines))
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
