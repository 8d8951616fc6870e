"""GPU parity at the full benchmark sizes (the launch configuration bench.py times), on sampled
query rows the fp64 oracle computes one by one against their complete key sets: per rollout
the first and last row, both sides of the prompt/response boundary and of every work-item
boundary, plus random rows; all heads.  Properties that hold at any size are checked on the
full tensors."""
import numpy as np
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import check, run_hip

pytestmark = pytest.mark.gpu


def sampled_parity(name, n_random, stride):
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    print(f"{name}: T={x.total_suffix} P={w.prefix_len} lens={x.suffix_lens.tolist()}", flush=True)
    out, lse = run_hip(x)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    rows = wl.sample_rows(x.suffix_lens, w.prompt_len, stride, n_random, seed=7)
    ro, rl, threads = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                   x.suffix_lens, w.scale, rows=rows)
    print(f"{name}: oracle on {len(rows)} rows x {w.num_q_heads} heads with {threads} threads", flush=True)
    check(out[rows], lse[:, rows], ro, rl, name)
    return x, out, lse


def test_c3_sampled_rows_and_prefix_permutation_property():
    x, out, lse = sampled_parity("C3", n_random=8, stride=64)
    # Property that holds at any size: the prefix rectangle has no order, so permuting the prefix
    # tokens (K and V together) may only change the floating-point summation order.
    perm = np.random.default_rng(5).permutation(x.workload.prefix_len)
    for n in ("k_prefix", "v_prefix"):
        x.bits[n] = np.ascontiguousarray(x.bits[n][perm])
    out2, lse2 = run_hip(x)
    d, dl = np.abs(out - out2), np.abs(lse - lse2)
    print(f"C3 prefix permutation: out max {d.max():.3e} mean {d.mean():.3e} lse max {dl.max():.3e}", flush=True)
    assert d.max() <= 2e-2 and d.mean() <= 1e-3 and dl.max() <= 1e-4


def test_c3_prefix_only_offset_sampled_rows():
    sampled_parity("C3pre", n_random=8, stride=64)


def test_c4_hour_long_sampled_rows():
    sampled_parity("C4", n_random=4, stride=576)


def test_c5_max_frames_ragged_sampled_rows():
    x, out, lse = sampled_parity("C5", n_random=2, stride=1024)
    assert len(set(x.suffix_lens.tolist())) > 8   # really ragged


def test_n1_prefix_self_attention_sampled_rows():
    """Causal self-attention of the 32K-token video prefix (P = 0, one sequence): the same library
    call, exercised as one long packed sequence whose rows cross hundreds of work items."""
    sampled_parity("N1", n_random=64, stride=4096)
