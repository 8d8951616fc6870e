"""Pins for the backward oracle (numpy definition and plain-C version), CPU only.

The backward is the derivative of the forward definition, so it is pinned to things that do
not share its formula: central finite differences of the forward oracle, torch autograd on
the concatenated per-rollout sequences, closed forms and invariants.  Planted mistakes
(dropped softmax-Jacobian term, missing scale, prefix gradient not summed over rollouts,
GQA group not summed, swapped K/V roles) must each fail the finite-difference pin.
"""
import numpy as np
import pytest

from oracle import cref
from oracle import ref_attention as ref
from paper_2507_07966_amd import workloads as wl

NAMES = ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")


def tiny(seed=0, Hq=4, Hkv=2, D=8, P=5, lens=(3, 1, 4)):
    x = wl.make_custom("f32", Hq, Hkv, D, P, lens, seed=seed)
    rng = np.random.default_rng(seed + 100)
    return x, rng.standard_normal(x.q.shape).astype(np.float32)


def bwd_np(x, do, scale):
    return ref.prefix_shared_attention_backward(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                x.suffix_lens, scale, do)


def bwd_c(x, do, scale):
    return cref.prefix_shared_attention_backward(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                 x.suffix_lens, scale, do)[:5]


IMPLS = [pytest.param(bwd_np, id="numpy"), pytest.param(bwd_c, id="c")]


def objective(arrs, lens, scale, do):
    out, _ = ref.prefix_shared_attention(arrs["q"], arrs["k_prefix"], arrs["v_prefix"], arrs["k_suffix"],
                                         arrs["v_suffix"], lens, scale)
    return float((out * do.astype(np.float64)).sum())


def finite_difference_gradients(x, do, scale, eps=1e-5):
    """dL/d(input) by central differences of the FORWARD oracle, one element at a time."""
    arrs = {n: np.array(getattr(x, n), dtype=np.float64) for n in NAMES}
    grads = {}
    for n in NAMES:
        g = np.zeros_like(arrs[n])
        flat, gflat = arrs[n].reshape(-1), g.reshape(-1)
        for e in range(flat.size):
            keep = flat[e]
            flat[e] = keep + eps
            up = objective(arrs, x.suffix_lens, scale, do)
            flat[e] = keep - eps
            dn = objective(arrs, x.suffix_lens, scale, do)
            flat[e] = keep
            gflat[e] = (up - dn) / (2 * eps)
        grads[n] = g
    return grads


def max_rel(a, b):
    return float(np.abs(a - b).max() / max(np.abs(b).max(), 1e-30))


# ---- B1: equals the numerical derivative of the forward oracle, every element of every input
@pytest.mark.parametrize("run", IMPLS)
def test_b1_matches_finite_differences_of_forward(run):
    x, do = tiny()
    fd = finite_difference_gradients(x, do, 0.4)
    got = run(x, do, 0.4)
    for n, g in zip(NAMES, got):
        assert g.shape == fd[n].shape
        assert max_rel(g, fd[n]) < 1e-7, n


# ---- B2: torch autograd (fp64) on the concatenated [prefix | suffix_g] sequences, prefix shared as one leaf
@pytest.mark.parametrize("run", IMPLS)
def test_b2_matches_torch_autograd(run):
    import torch
    x, do = tiny(seed=3, Hq=6, Hkv=2, D=16, P=11, lens=(7, 2, 9))
    scale = 0.25
    t = {n: torch.tensor(np.asarray(getattr(x, n), dtype=np.float64), requires_grad=True) for n in NAMES}
    P, r = 11, 3
    off = ref.suffix_offsets(x.suffix_lens)
    loss = torch.zeros((), dtype=torch.float64)
    for g, S in enumerate(x.suffix_lens):
        a, b = int(off[g]), int(off[g + 1])
        keys = torch.cat([t["k_prefix"], t["k_suffix"][a:b]], 0).repeat_interleave(r, dim=1)   # [P+S, Hq, D]
        vals = torch.cat([t["v_prefix"], t["v_suffix"][a:b]], 0).repeat_interleave(r, dim=1)
        mask = torch.ones(S, P + S, dtype=torch.bool)
        mask[:, P:] = torch.tril(torch.ones(S, S, dtype=torch.bool))
        o = torch.nn.functional.scaled_dot_product_attention(
            t["q"][a:b].transpose(0, 1), keys.transpose(0, 1), vals.transpose(0, 1), attn_mask=mask, scale=scale)
        loss = loss + (o.transpose(0, 1) * torch.tensor(do[a:b], dtype=torch.float64)).sum()
    loss.backward()
    got = run(x, do, scale)
    for n, g in zip(NAMES, got):
        assert max_rel(g, t[n].grad.numpy()) < 1e-10, n


# ---- B3: a row that sees one key has weight 1: no gradient reaches q or k, dv = sum of dO over the group
@pytest.mark.parametrize("run", IMPLS)
def test_b3_single_visible_key(run):
    x, do = tiny(seed=4, Hq=4, Hkv=2, D=8, P=0, lens=(1, 1))
    dq, dkp, dvp, dks, dvs = run(x, do, 0.7)
    assert np.abs(dq).max() < 1e-14 and np.abs(dks).max() < 1e-14
    assert dkp.shape == (0, 2, 8) and dvp.shape == (0, 2, 8)
    want = do.astype(np.float64).reshape(2, 2, 2, 8).sum(axis=2)     # [token, kv head, D]
    assert np.abs(dvs - want).max() < 1e-14


# ---- B4: zero queries: weights are uniform, dk = 0, dv_j = sum over seeing rows of dO / n_visible,
#          dq = scale * sum_j (1/n) (dW_j - mean dW) k_j
@pytest.mark.parametrize("run", IMPLS)
def test_b4_uniform_weights_closed_form(run):
    x, do = tiny(seed=5, Hq=2, Hkv=1, D=8, P=3, lens=(4,))
    x.q[...] = 0
    scale = 0.9
    dq, dkp, dvp, dks, dvs = run(x, do, scale)
    assert np.abs(dkp).max() < 1e-14 and np.abs(dks).max() < 1e-14
    do64 = do.astype(np.float64)
    want_vp = np.zeros((3, 8))
    want_vs = np.zeros((4, 8))
    for i in range(4):
        n = 3 + i + 1
        for h in range(2):
            want_vp += do64[i, h] / n
            want_vs[:i + 1] += do64[i, h] / n
            keys = np.concatenate([x.k_prefix[:, 0], x.k_suffix[:i + 1, 0]]).astype(np.float64)
            vals = np.concatenate([x.v_prefix[:, 0], x.v_suffix[:i + 1, 0]]).astype(np.float64)
            dw = vals @ do64[i, h]
            want_q = scale * ((dw - dw.mean()) / n) @ keys
            assert np.abs(dq[i, h] - want_q).max() < 1e-13
    assert np.abs(dvp[:, 0] - want_vp).max() < 1e-13
    assert np.abs(dvs[:, 0] - want_vs).max() < 1e-13


# ---- B5: invariants that hold for any input
@pytest.mark.parametrize("run", IMPLS)
def test_b5_invariants(run):
    def grid_keys():       # keys on a 1/16 grid, so that the shift below is exact in fp32
        y, d = tiny(seed=6, Hq=6, Hkv=2, D=8, P=9, lens=(5, 3, 8))
        y.k_prefix[...] = np.round(y.k_prefix * 16) / 16
        y.k_suffix[...] = np.round(y.k_suffix * 16) / 16
        return y, d

    x, do = grid_keys()
    dq, dkp, dvp, dks, dvs = run(x, do, 0.35)
    do64 = do.astype(np.float64)
    for c in range(2):
        hs = slice(3 * c, 3 * c + 3)
        # every row's weights sum to one, so the value gradients of a kv head sum to its rows' dO
        assert np.abs(dvp[:, c].sum(0) + dvs[:, c].sum(0) - do64[:, hs].sum((0, 1))).max() < 1e-12
        # <q, dq> and <k, dk> are the same contraction of dS with the scores
        lhs = (x.q[:, hs].astype(np.float64) * dq[:, hs]).sum()
        rhs = (x.k_prefix[:, c].astype(np.float64) * dkp[:, c]).sum() + (x.k_suffix[:, c].astype(np.float64) * dks[:, c]).sum()
        assert abs(lhs - rhs) < 1e-12 * max(1.0, abs(lhs))
    # shifting every key by the same vector moves all scores of a row together: no weight changes, and
    # because every row of dS sums to zero, dq does not change either
    x2, _ = grid_keys()
    mu = (np.arange(8, dtype=np.float32) - 3) / 4
    x2.k_prefix += mu
    x2.k_suffix += mu
    dq2 = run(x2, do, 0.35)[0]
    assert np.abs(dq2 - dq).max() < 1e-12


# ---- B6: rollouts interact only through the shared prefix: the prefix gradients are the sum of
#          the single-rollout gradients, the suffix gradients are the single-rollout ones
@pytest.mark.parametrize("run", IMPLS)
def test_b6_prefix_gradient_is_sum_over_rollouts(run):
    x, do = tiny(seed=7, Hq=4, Hkv=2, D=8, P=6, lens=(4, 2, 5))
    dq, dkp, dvp, dks, dvs = run(x, do, 0.5)
    off = ref.suffix_offsets(x.suffix_lens)
    acc_k, acc_v = np.zeros_like(dkp), np.zeros_like(dvp)
    for g, S in enumerate(x.suffix_lens):
        a, b = int(off[g]), int(off[g + 1])
        one = wl.make_custom("f32", 4, 2, 8, 6, (int(S),), seed=0)
        one.q, one.k_suffix, one.v_suffix = x.q[a:b], x.k_suffix[a:b], x.v_suffix[a:b]
        one.k_prefix, one.v_prefix = x.k_prefix, x.v_prefix
        q1, kp1, vp1, ks1, vs1 = run(one, do[a:b], 0.5)
        acc_k += kp1
        acc_v += vp1
        assert np.abs(q1 - dq[a:b]).max() < 1e-13
        assert np.abs(ks1 - dks[a:b]).max() < 1e-13 and np.abs(vs1 - dvs[a:b]).max() < 1e-13
    assert np.abs(acc_k - dkp).max() < 1e-12 and np.abs(acc_v - dvp).max() < 1e-12


def test_c_backward_equals_numpy_definition_and_row_subset():
    x = wl.make_custom("bf16", 14, 2, 64, 70, (33, 1, 64, 17), seed=8)
    do = np.random.default_rng(9).standard_normal(x.q.shape).astype(np.float32)
    a = bwd_np(x, do, x.workload.scale)
    b = bwd_c(x, do, x.workload.scale)
    for n, u, v in zip(NAMES, a, b):
        assert np.abs(u - v).max() < 1e-12, n
    rows = np.array([0, 32, 33, 34, 97, 114])
    dq_rows, _ = cref.prefix_shared_attention_backward(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                       x.suffix_lens, x.workload.scale, do, rows=rows)
    assert np.abs(dq_rows - a[0][rows]).max() < 1e-12


def test_planted_backward_mistakes_fail_the_finite_difference_pin():
    """The finite-difference pin must tell a correct backward from plausible wrong ones."""
    x, do = tiny()
    scale = 0.4
    fd = finite_difference_gradients(x, do, scale)
    good = dict(zip(NAMES, bwd_np(x, do, scale)))

    def differs(name, arr):
        return max_rel(arr, fd[name]) > 1e-3

    off = ref.suffix_offsets(x.suffix_lens)
    P, r = 5, 2
    # (1) softmax Jacobian without the row-sum term, (2) no scale on dq, (3) prefix gradient from the last
    # rollout only, (4) kv-head gradient from one q head of the group only, (5) dv built from dS instead of W
    no_delta = np.zeros_like(good["q"])
    last_only = np.zeros_like(good["k_prefix"])
    one_head = np.zeros_like(good["v_suffix"])
    dv_from_ds = np.zeros_like(good["v_prefix"])
    for g in range(len(x.suffix_lens)):
        a, b = int(off[g]), int(off[g + 1])
        for h in range(4):
            c = h // r
            w, _ = ref.attention_weights(x.q, x.k_prefix, x.k_suffix, x.suffix_lens, scale, g, h)
            keys = np.concatenate([x.k_prefix[:, c], x.k_suffix[a:b, c]]).astype(np.float64)
            vals = np.concatenate([x.v_prefix[:, c], x.v_suffix[a:b, c]]).astype(np.float64)
            d = do[a:b, h].astype(np.float64)
            dw = d @ vals.T
            ds = w * (dw - (w * dw).sum(1, keepdims=True))
            no_delta[a:b, h] = scale * ((w * dw) @ keys)
            dkeys = scale * ds.T @ x.q[a:b, h].astype(np.float64)
            if g == len(x.suffix_lens) - 1:
                last_only[:, c] += dkeys[:P]
            if h % r == 0:
                one_head[a:b, c] += (w.T @ d)[P:]
            dv_from_ds[:, c] += (ds.T @ d)[:P]
    assert differs("q", no_delta)
    assert differs("q", good["q"] / scale)
    assert differs("k_prefix", last_only)
    assert differs("v_suffix", one_head)
    assert differs("v_prefix", dv_from_ds)
    assert differs("k_suffix", good["v_suffix"])
    for n in NAMES:
        assert not differs(n, good[n])


@pytest.mark.parametrize("run", IMPLS)
def test_hand_worked_backward_golden(run):
    import json
    import os
    cases = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked_backward_logprob.json")))["backward_cases"]
    for c in cases:
        x = wl.make_custom("f32", 1, 1, 1, 1, c["suffix_lens"], seed=0)
        for n in NAMES:
            setattr(x, n, np.array(c[n], dtype=np.float32))
        got = run(x, np.array(c["d_out"], dtype=np.float32), c["scale"])
        for n, g in zip(("dq", "dk_prefix", "dv_prefix", "dk_suffix", "dv_suffix"), got):
            assert np.abs(g - np.array(c[n])).max() < 1e-6, (c["name"], n)     # inputs are fp32-rounded (ln 3 as scale is exact in fp64)
