"""Build libprefix_attn.so (C-ABI library, gfx950) in-tree with hipcc.

Run `python -m paper_2507_07966_amd.build`.  hipcc cross-compiles without a GPU.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libprefix_attn.so")
SOURCES = ["plan.cpp", "api.cpp", "attn_bf16.hip", "attn_f32.hip", "vt_image.hip", "merge.hip",
           "bwd_api.cpp", "bwd_prep.hip", "bwd_dq_bf16.hip", "bwd_dkv_bf16.hip", "bwd_f32.hip",
           "logprob_api.cpp", "logprob.hip"]
# packed-fp32 code generation is switched off for every device translation unit
DEVICE_FLAGS = ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                # MFMA results in ordinary vector registers; kernels that need more than 256 registers keep
                # long-lived MFMA operands in the accumulation registers instead (see bwd_dkv_bf16.hip)
                "-mllvm", "-amdgpu-mfma-vgpr-form=1"]


def build(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    bdir = os.path.join(HERE, "_build", os.path.basename(out))
    os.makedirs(bdir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src + ".o")
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-x", "hip", *DEVICE_FLAGS,
               "-Wall", "-Wno-unused-command-line-argument", f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}",
               *extra_flags, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        log, _ = p.communicate()
        log = "\n".join(l for l in log.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{log}", file=sys.stderr)
        elif log.strip() and verbose:
            print(log)
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
