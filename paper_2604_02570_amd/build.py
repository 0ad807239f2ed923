"""Build libwsvd.so (gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libwsvd.so")
LIB_TIMELINE = os.path.join(HERE, "libwsvd_timeline.so")     # profiling build: in-kernel wall-clock stamps compiled in
SOURCES = ["wsvd_api.hip", "wsvd_quant.hip", "wsvd_append.hip", "wsvd_attn_generic.hip", "wsvd_attn_mfma.hip",
           "wsvd_block.hip", "wsvd_layer.hip", "wsvd_prefill.hip", "wsvd_project.hip", "wsvd_shared.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]
# per-file additions.  The prompt attention reads every score tile back into the vector ALU, which binds it: its matrix
# products write ordinary vector registers instead of accumulation registers (no copies between the two files).
FILE_FLAGS = {"wsvd_prefill.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def build(verbose: bool = True, extra_flags=(), timeline: bool = False) -> str:
    """Compile every source for gfx950 and link libwsvd.so; timeline=True builds the profiling variant
    libwsvd_timeline.so (-DWSVD_TIMELINE) beside it instead."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build", "timeline" if timeline else "product")
    lib_path = LIB_TIMELINE if timeline else LIB
    if timeline:
        extra_flags = (*extra_flags, "-DWSVD_TIMELINE")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        cmd = [hipcc, *FLAGS, *FILE_FLAGS.get(src, []), *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, obj, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    objs = []
    for src, obj, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{out}")
        if verbose and out.strip():
            print(out)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", lib_path]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}")
    if verbose:
        print(f"built {lib_path}")
    return lib_path


if __name__ == "__main__":
    argv = sys.argv[1:]
    tl = "--timeline" in argv
    build(extra_flags=[a for a in argv if a != "--timeline"], timeline=tl)
