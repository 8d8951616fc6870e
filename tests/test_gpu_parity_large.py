"""GPU parity at the full benchmark sizes (the launch configuration bench.py times), on sampled
query rows the fp64 oracle computes one by one against their complete key sets: per rollout
the first and last row, both sides of the prompt/response boundary and of multiples of the key
tile, the positions around work-item boundaries (every 256 stacked rows = 256/7 positions: all
of them at the graded 32K-prefix configuration, a seeded subset at the larger ones, where a row
costs the oracle 7 to 16 times more), plus random rows; all heads.  Properties that hold at any
size are checked on the full tensors.  The graded code path is also compared element by element
on a smaller full tensor in tests/test_gpu_parity.py."""
import numpy as np
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import check, run_hip

pytestmark = pytest.mark.gpu


def sampled_parity(name, n_random, stride, item_bounds=None):
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    print(f"{name}: T={x.total_suffix} P={w.prefix_len} lens={x.suffix_lens.tolist()}", flush=True)
    out, lse = run_hip(x)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    rows = wl.sample_rows(x.suffix_lens, w.prompt_len, stride, n_random, seed=7,
                          group=w.num_q_heads // w.num_kv_heads, item_bounds=item_bounds)
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
    sampled_parity("C3pre", n_random=8, stride=64, item_bounds=8)


def test_c4_hour_long_sampled_rows():
    sampled_parity("C4", n_random=4, stride=576, item_bounds=4)


def test_c5_max_frames_ragged_sampled_rows():
    x, out, lse = sampled_parity("C5", n_random=1, stride=4096, item_bounds=1)
    assert len(set(x.suffix_lens.tolist())) > 8   # really ragged


def test_n1_prefix_self_attention_sampled_rows():
    """Causal self-attention of the 32K-token video prefix (P = 0, one sequence): the same library
    call, exercised as one long packed sequence whose rows cross hundreds of work items."""
    sampled_parity("N1", n_random=64, stride=4096, item_bounds=24)


def test_n1h_hour_long_prefix_self_attention_sampled_rows():
    """230,400 video tokens in one causal sequence (6,300 work items per kv head, 3.8e14 FLOP)."""
    sampled_parity("N1h", n_random=24, stride=65536, item_bounds=8)


@pytest.mark.parametrize("name,stride,n_random,item_bounds", [("C3", 256, 4, 2), ("C4", 1 << 20, 1, 1)])
def test_backward_sampled_rows_and_invariants(name, stride, n_random, item_bounds):
    """Backward at the full 32K-prefix and hour-long (230K-prefix) sizes.  dQ is checked on sampled rows the
    oracle computes one by one.  dK/dV of a prefix key sum over all 516,096 (row, head) pairs, which the oracle
    cannot afford here, so they are checked through two identities that hold at any size (both pinned on the
    oracle):
      sum over keys of dV = sum over rows of dO            (every row's weights sum to one)
      <q, dq> = <k, dk>                                     (both contract dS with the scores)
    and element by element, on the same direct (one item per key block, several rounds) dK/dV path, on a
    16K-prefix case in tests/test_gpu_backward.py."""
    from tests.gpu_util import check_grad_tensor, run_hip_backward
    w = wl.WORKLOADS[name]
    x = wl.make_inputs(w)
    do, bits = wl.make_d_out(x)
    got = run_hip_backward(x, do, bits)
    for n, a in got.items():
        assert np.isfinite(a).all(), n
    r = w.num_q_heads // w.num_kv_heads
    rows = wl.sample_rows(x.suffix_lens, w.prompt_len, stride, n_random, seed=11, group=r, item_bounds=item_bounds)
    dq_ref, threads = cref.prefix_shared_attention_backward(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                            x.suffix_lens, w.scale, do, rows=rows)
    check_grad_tensor(got["dq"][rows], dq_ref, "bf16", f"{name} backward dq on {len(rows)} rows")
    u = 2.0 ** -9      # relative rounding of a bf16 result
    for c in range(w.num_kv_heads):
        hs = slice(c * r, (c + 1) * r)
        # value gradients: sum over all keys against the sum of dO over the head group's rows
        lhs = got["dv_prefix"][:, c].sum(0) + got["dv_suffix"][:, c].sum(0)
        rhs = do[:, hs].astype(np.float64).sum((0, 1))
        n_keys = got["dv_prefix"].shape[0] + got["dv_suffix"].shape[0]
        el = max(float(np.sqrt(np.mean(got["dv_prefix"][:, c] ** 2))), float(np.sqrt(np.mean(got["dv_suffix"][:, c] ** 2))))
        tol = 16 * np.sqrt(n_keys) * u * el         # independent roundings of n_keys outputs, generous factor
        print(f"{name} backward kv head {c}: |sum dV - sum dO| max {np.abs(lhs - rhs).max():.3e} (tol {tol:.3e}, "
              f"|sum| rms {np.sqrt(np.mean(rhs * rhs)):.3e})", flush=True)
        assert np.sqrt(np.mean(rhs * rhs)) > 20 * tol      # the identity is not vacuous at this tolerance
        assert np.abs(lhs - rhs).max() <= tol
        # key/query gradients
        qd = x.q[:, hs].astype(np.float64) * got["dq"][:, hs]
        kd_p = x.k_prefix[:, c].astype(np.float64) * got["dk_prefix"][:, c]
        kd_s = x.k_suffix[:, c].astype(np.float64) * got["dk_suffix"][:, c]
        a, b = qd.sum(), kd_p.sum() + kd_s.sum()
        tol2 = 8 * u * np.sqrt((qd ** 2).sum() + (kd_p ** 2).sum() + (kd_s ** 2).sum())
        print(f"{name} backward kv head {c}: <q,dq> {a:.4f} <k,dk> {b:.4f} (tol {tol2:.3e})", flush=True)
        assert abs(a - b) <= tol2


def test_c5_backward_ragged_sampled_dq_rows_and_value_identity():
    """Backward at the largest configuration (512K prefix keys, 16 ragged rollouts): dQ on sampled rows against
    the oracle, and the value-gradient identity sum_keys dV = sum_rows dO on the full tensors."""
    from tests.gpu_util import check_grad_tensor, run_hip_backward
    w = wl.WORKLOADS["C5"]
    x = wl.make_inputs(w)
    do, bits = wl.make_d_out(x)
    got = run_hip_backward(x, do, bits)
    for n, a in got.items():
        assert np.isfinite(a).all(), n
    # first/last/prompt boundary + 1 random per rollout; every other one of them (a row costs the oracle 1.1e10 FLOP)
    rows = wl.sample_rows(x.suffix_lens, w.prompt_len, 1 << 20, 1, seed=13)[::2]
    dq_ref, _ = cref.prefix_shared_attention_backward(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                      x.suffix_lens, w.scale, do, rows=rows)
    check_grad_tensor(got["dq"][rows], dq_ref, "bf16", f"C5 backward dq on {len(rows)} rows")
    r = w.num_q_heads // w.num_kv_heads
    for c in range(w.num_kv_heads):
        lhs = got["dv_prefix"][:, c].sum(0) + got["dv_suffix"][:, c].sum(0)
        rhs = do[:, c * r:(c + 1) * r].astype(np.float64).sum((0, 1))
        n_keys = got["dv_prefix"].shape[0] + got["dv_suffix"].shape[0]
        el = max(float(np.sqrt(np.mean(got["dv_prefix"][:, c] ** 2))), float(np.sqrt(np.mean(got["dv_suffix"][:, c] ** 2))))
        tol = 16 * np.sqrt(n_keys) * 2.0 ** -9 * el       # as in the C3 test; the sums themselves are of order 500
        print(f"C5 backward kv head {c}: |sum dV - sum dO| max {np.abs(lhs - rhs).max():.3e} (tol {tol:.3e})", flush=True)
        assert np.abs(lhs - rhs).max() <= tol


def test_c3_shared_question_folded_into_the_prefix_sampled_rows():
    """Two-level sharing at the 32K-prefix shape: the prompt-only call (28 blocks of rows: its prefix keys are
    split into 9 ranges) and the call with prefix 33,024 against the oracle's plain per-rollout definition."""
    from tests.fold_util import unfold_rows
    w = wl.WORKLOADS["C3"]
    x = wl.share_prompt(wl.make_inputs(w))
    p, f, where = wl.fold_prompt(x)
    po, pl = run_hip(p)
    fo, fl = run_hip(f)
    rows = wl.sample_rows(x.suffix_lens, w.prompt_len, 256, 4, seed=17)
    ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                             w.scale, rows=rows)
    out = unfold_rows(where[rows], fo, po)
    lse = unfold_rows(where[rows], fl.T, pl.T).T
    check(out, lse, ro, rl, "C3 two-level")
