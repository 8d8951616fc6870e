"""Pins of the oracle against a grouping invariance (CPU only): when the G rollouts share their prompt
(same question, Sec. 4.2), attention over [video | prompt | response_g] per rollout must equal the
two-level arrangement that computes the prompt once and treats [video | prompt] as the shared prefix.
Forward: the same rows.  Backward: gradients of shared tokens are the sums over the rollouts' copies.
A wrong mask boundary, a wrong prefix/suffix offset or a dropped sum over rollouts breaks one of these."""
import numpy as np
import pytest

from oracle import cref, ref_attention as ref
from paper_2507_07966_amd import workloads as wl
from tests.fold_util import args, folded_backward, unfold_rows, unfolded_backward


def small(dtype="f32", seed=5):
    w = wl.Workload("fold", dtype, 4, 2, 16, 6, 4, 5, 3, None, response_range=(2, 9), seed=seed)
    return wl.share_prompt(wl.make_inputs(w))


def test_fold_is_a_rearrangement_only():
    x = small("bf16")
    p, f, rows = wl.fold_prompt(x)
    Lp, P = x.workload.prompt_len, x.workload.prefix_len
    assert p.workload.prefix_len == P and list(p.suffix_lens) == [Lp]
    assert f.workload.prefix_len == P + Lp and (f.suffix_lens == x.suffix_lens - Lp).all()
    assert np.array_equal(unfold_rows(rows, f.q, p.q), x.q)
    assert np.array_equal(unfold_rows(rows, f.bits["k_suffix"], p.bits["k_suffix"]), x.bits["k_suffix"])
    assert np.array_equal(f.v_prefix[:P], x.v_prefix) and np.array_equal(f.v_prefix[P:], x.v_suffix[:Lp])


def test_forward_equals_two_level_arrangement():
    x = small()
    p, f, rows = wl.fold_prompt(x)
    out, lse = ref.prefix_shared_attention(*args(x))
    po, pl = ref.prefix_shared_attention(*args(p))
    fo, fl = ref.prefix_shared_attention(*args(f))
    np.testing.assert_allclose(unfold_rows(rows, fo, po), out, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(unfold_rows(rows, fl.T, pl.T).T, lse, rtol=1e-12, atol=1e-13)


def numpy_backward(x, d_out):
    return ref.prefix_shared_attention_backward(*args(x), d_out)


def c_backward(x, d_out):
    return cref.prefix_shared_attention_backward(*args(x), d_out)[:5]


def test_backward_equals_two_level_arrangement_numpy():
    x = small()
    d_out, _ = wl.make_d_out(x)
    a = unfolded_backward(numpy_backward, x, d_out)
    b = folded_backward(numpy_backward, x, d_out)
    for n in a:
        np.testing.assert_allclose(b[n], a[n], rtol=1e-11, atol=1e-12, err_msg=n)


def test_two_level_arrangement_c_oracle_ragged_bf16_values():
    w = wl.Workload("fold", "bf16", 8, 2, 64, 9, 16, 37, 4, None, response_range=(20, 150), seed=9)
    x = wl.share_prompt(wl.make_inputs(w))
    p, f, rows = wl.fold_prompt(x)
    out, lse, _ = cref.prefix_shared_attention(*args(x))
    po, pl, _ = cref.prefix_shared_attention(*args(p))
    fo, fl, _ = cref.prefix_shared_attention(*args(f))
    np.testing.assert_allclose(unfold_rows(rows, fo, po), out, rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(unfold_rows(rows, fl.T, pl.T).T, lse, rtol=1e-10, atol=1e-11)
    d_out, _ = wl.make_d_out(x, grid=1 / 8)          # the C oracle takes fp32 inputs: keep the summed dO exact
    a = unfolded_backward(c_backward, x, d_out)
    b = folded_backward(c_backward, x, d_out)
    for n in a:
        np.testing.assert_allclose(b[n], a[n], rtol=1e-9, atol=1e-10, err_msg=n)


def test_planted_mistake_prompt_gradient_without_rollout_sum_is_caught():
    x = small()
    d_out, _ = wl.make_d_out(x)
    a = unfolded_backward(numpy_backward, x, d_out)
    p, f, rows = wl.fold_prompt(x)
    wrong = ref.prefix_shared_attention_backward(*args(p), d_out[:x.workload.prompt_len])[0]   # rollout 0's dO only
    assert not np.allclose(wrong, a["dq_prompt"], rtol=1e-3, atol=1e-6)
