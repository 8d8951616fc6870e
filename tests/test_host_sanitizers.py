"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, on the CPU.

(1) The library's host side (plan building, schedule introspection, argument checks of every entry point:
plan.cpp, api.cpp, bwd_api.cpp, logprob_api.cpp) is compiled with hipcc, the sanitizers applied to the
host pass only, together with stand-ins for the kernel launchers and a native driver that goes through the
C ABI with host-only plans (tests/native/abi_driver.cpp).
(2) The fp64 C oracle is compiled with gcc and the same sanitizers into a driver program
(tests/native/oracle_driver.c); its results on ragged cases (forward, backward, row subsets, no prefix)
must equal those of the ordinary build.
Both are separate programs, so the test interpreter itself needs no sanitizer runtime."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
CSRC = os.path.join(ROOT, "paper_2507_07966_amd", "csrc")
SAN_ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def run(cmd, **kw):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, **kw)
    assert r.returncode == 0, f"{' '.join(cmd)}\n{r.stdout[-4000:]}"
    return r.stdout


def test_library_host_side_under_sanitizers(tmp_path):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    exe = str(tmp_path / "abi_driver")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]
    srcs = [os.path.join(CSRC, f) for f in ("plan.cpp", "api.cpp", "bwd_api.cpp", "logprob_api.cpp")]
    srcs += [os.path.join(NATIVE, "launch_stubs.cpp"), os.path.join(NATIVE, "abi_driver.cpp")]
    run([hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-x", "hip", *san, "-Wno-unused-command-line-argument",
         f"-I{os.path.join(ROOT, 'include')}", f"-I{CSRC}", *srcs, "-o", exe])
    out = run([exe], env=SAN_ENV)
    assert "abi_driver: ok" in out, out


def write_case(path, x, scale, d_out=None, rows=None):
    w = x.workload
    with open(path, "wb") as f:
        np.array([len(x.suffix_lens), w.prefix_len, w.num_q_heads, w.num_kv_heads, w.head_dim,
                  0 if rows is None else len(rows), int(d_out is not None), 0], dtype=np.int64).tofile(f)
        np.array([scale], dtype=np.float64).tofile(f)
        x.suffix_lens.astype(np.int32).tofile(f)
        for a in (x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix):
            np.ascontiguousarray(a, dtype=np.float32).tofile(f)
        if d_out is not None:
            np.ascontiguousarray(d_out, dtype=np.float32).tofile(f)
        if rows is not None:
            np.ascontiguousarray(rows, dtype=np.int64).tofile(f)


def test_c_oracle_under_sanitizers(tmp_path):
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("gcc not found")
    exe = str(tmp_path / "oracle_driver")
    run([gcc, "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", os.path.join(ROOT, "oracle", "ref_attention.c"),
         os.path.join(NATIVE, "oracle_driver.c"), "-o", exe, "-lm"])
    cases = [("bf16", 6, 2, 64, 37, (5, 1, 19)), ("f32", 4, 4, 128, 0, (9, 2)), ("bf16", 7, 1, 64, 1, (1,))]
    for i, (dtype, Hq, Hkv, D, P, lens) in enumerate(cases):
        x = wl.make_custom(dtype, Hq, Hkv, D, P, lens, seed=50 + i)
        do, _ = wl.make_d_out(x)
        T = x.total_suffix
        a = (x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, 0.17)
        rows = np.array(sorted({0, T - 1, T // 2}), dtype=np.int64)
        for tag, d_out, rr in (("fwd", None, None), ("fwd_rows", None, rows), ("bwd", do, None), ("bwd_rows", do, rows)):
            fin, fout = str(tmp_path / f"case{i}_{tag}.in"), str(tmp_path / f"case{i}_{tag}.out")
            write_case(fin, x, 0.17, d_out, rr)
            run([exe, fin, fout], env=dict(SAN_ENV, OMP_NUM_THREADS="3"))
            got = np.fromfile(fout, dtype=np.float64)
            if d_out is None:
                o, l, _ = cref.prefix_shared_attention(*a, rows=rr)
                want = np.concatenate([o.ravel(), l.ravel()])
            else:
                res = cref.prefix_shared_attention_backward(*a, d_out, rows=rr)
                want = np.concatenate([r.ravel() for r in res[:-1]])
            assert got.shape == want.shape, (tag, got.shape, want.shape)
            assert np.abs(got - want).max() <= 1e-12 * max(1.0, np.abs(want).max()), tag
