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


# hipcc hands the target-feature flag to its host pass as well, which does not know it and says so once per
# translation unit.  Only that exact line is dropped from the logs, and only after check_device_flag() has
# shown that the device pass accepts the flag silently.
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def check_device_flag(hipcc: str, bdir: str) -> None:
    """Compile a one-line kernel for the device only: the device pass must take the flags without comment."""
    src = os.path.join(bdir, "flag_probe.hip")
    with open(src, "w") as f:
        f.write("__global__ void flag_probe(float* p) { p[0] = 1.f; }\n")
    r = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-x", "hip", *DEVICE_FLAGS, "--cuda-device-only", "-c",
                        src, "-o", os.path.join(bdir, "flag_probe.o")], stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0 or "packed-fp32-ops" in r.stdout:
        raise RuntimeError(f"the device compilation pass does not accept the build's flags:\n{r.stdout}")


def build(verbose: bool = False, extra_flags=(), out: str = LIB) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    bdir = os.path.join(HERE, "_build", os.path.basename(out))
    os.makedirs(bdir, exist_ok=True)
    check_device_flag(hipcc, bdir)
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
        log = "\n".join(l for l in log.splitlines() if l.strip() != HOST_PASS_NOTE)
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


PROBE = os.path.join(HERE, "power_probe")


def build_probe(out: str = PROBE) -> str:
    """The stand-alone measurement program csrc/power_probe.hip (MFMA rate under the power limit, with and without
    LDS operand reads): not part of the library, built beside it so that its record under profiles/ can be re-made."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", *DEVICE_FLAGS[:4], "-Wall",
           "-Wno-unused-command-line-argument", os.path.join(CSRC, "power_probe.hip"), "-o", out]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log = "\n".join(l for l in r.stdout.splitlines() if l.strip() != HOST_PASS_NOTE)
    if r.returncode != 0:
        print(f"[build] power_probe.hip FAILED\n{log}", file=sys.stderr)
        raise RuntimeError("hipcc failed")
    return out


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv))
    print(build_probe())
