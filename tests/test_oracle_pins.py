"""Pins for the fp64 oracle (numpy definition and plain-C version), CPU only.

The paper prints no worked numeric attention example, so the oracle is pinned by
closed forms, invariants, brute force on tiny inputs and one library routine.
Each pin is chosen so that a dropped term, a wrong sign/index, a transposed
operand or a wrong head mapping fails at least one of them.
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import cref
from oracle import ref_attention as ref
from paper_2507_07966_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(seed=0, Hq=4, Hkv=2, D=8, P=5, lens=(3, 1, 4), dtype="f32"):
    return wl.make_custom(dtype, Hq, Hkv, D, P, lens, seed=seed)


def run_np(x, scale=None):
    scale = x.workload.scale if scale is None else scale
    return ref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, scale)


def run_c(x, scale=None, rows=None):
    scale = x.workload.scale if scale is None else scale
    o, l, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                           x.suffix_lens, scale, rows=rows)
    return o, l


IMPLS = [pytest.param(run_np, id="numpy"), pytest.param(run_c, id="c")]


# ---- P1: weights are a probability distribution over exactly the visible keys
def test_p1_weights_nonneg_rows_sum_to_one_and_mask():
    x = tiny()
    P = x.workload.prefix_len
    for g, S in enumerate(x.suffix_lens):
        for h in range(4):
            w, _ = ref.attention_weights(x.q, x.k_prefix, x.k_suffix, x.suffix_lens, 0.3, g, h)
            assert w.shape == (S, P + S)
            assert (w >= 0).all()
            assert np.abs(w.sum(axis=1) - 1).max() < 1e-12
            for i in range(S):
                assert (w[i, P + i + 1:] == 0).all()      # future suffix tokens carry no weight
                assert (w[i, :P + i + 1] > 0).all()       # prefix and past+self all visible


# ---- P2: zero queries => arithmetic mean of visible V rows, LSE = ln(count)
@pytest.mark.parametrize("run", IMPLS)
def test_p2_uniform_scores_give_mean_of_v(run):
    x = tiny(seed=1)
    x.q[...] = 0
    out, lse = run(x)
    off = ref.suffix_offsets(x.suffix_lens)
    P = x.workload.prefix_len
    for g, S in enumerate(x.suffix_lens):
        for h in range(4):
            c = h // 2
            for i in range(S):
                vis = np.concatenate([x.v_prefix[:, c], x.v_suffix[off[g]:off[g] + i + 1, c]]).astype(np.float64)
                assert np.allclose(out[off[g] + i, h], vis.mean(axis=0), atol=1e-13)
                assert abs(lse[h, off[g] + i] - math.log(P + i + 1)) < 1e-13


# ---- P3: causality
@pytest.mark.parametrize("run", IMPLS)
def test_p3_later_tokens_do_not_matter(run):
    x = tiny(seed=2, lens=(6, 5))
    out0, lse0 = run(x)
    off = ref.suffix_offsets(x.suffix_lens)
    cut = 3
    rng = np.random.default_rng(9)
    for g in range(2):
        sl = slice(off[g] + cut, off[g + 1])
        for a in (x.q, x.k_suffix, x.v_suffix):
            a[sl] += rng.standard_normal(a[sl].shape).astype(np.float32)
    out1, lse1 = run(x)
    for g in range(2):
        keep = slice(off[g], off[g] + cut)
        assert np.array_equal(out0[keep], out1[keep])
        assert np.array_equal(lse0[:, keep], lse1[:, keep])
        changed = slice(off[g] + cut, off[g + 1])
        assert not np.array_equal(out0[changed], out1[changed])


# ---- P4: sharing the prefix == independent full-sequence attention per rollout (brute force loops)
@pytest.mark.parametrize("run", IMPLS)
def test_p4_equals_bruteforce_full_sequence(run):
    x = tiny(seed=3, Hq=4, Hkv=2, D=4, P=6, lens=(3, 5, 1))
    scale = 0.37
    out, lse = run(x, scale)
    off = ref.suffix_offsets(x.suffix_lens)
    rng = np.random.default_rng(5)
    P = 6
    for g, S in enumerate(x.suffix_lens):
        for h in range(4):
            c = h // 2
            q_full = np.concatenate([rng.standard_normal((P, 4)), x.q[off[g]:off[g + 1], h]])  # prefix queries arbitrary
            k_full = np.concatenate([x.k_prefix[:, c], x.k_suffix[off[g]:off[g + 1], c]])
            v_full = np.concatenate([x.v_prefix[:, c], x.v_suffix[off[g]:off[g + 1], c]])
            o_bf, l_bf = ref.full_causal_attention_bruteforce(q_full.tolist(), k_full.tolist(), v_full.tolist(), scale)
            assert np.abs(o_bf[P:] - out[off[g]:off[g + 1], h]).max() < 1e-12
            assert np.abs(l_bf[P:] - lse[h, off[g]:off[g + 1]]).max() < 1e-12


# ---- P5: library routine on the concatenated sequence
@pytest.mark.parametrize("run", IMPLS)
def test_p5_matches_torch_sdpa_float64(run):
    import torch
    x = tiny(seed=4, Hq=6, Hkv=2, D=16, P=33, lens=(17, 9))
    scale = x.workload.scale
    out, lse = run(x)
    off = ref.suffix_offsets(x.suffix_lens)
    P, r = 33, 3
    for g, S in enumerate(x.suffix_lens):
        k_full = torch.from_numpy(np.concatenate([x.k_prefix, x.k_suffix[off[g]:off[g + 1]]])).double()  # [L,Hkv,D]
        v_full = torch.from_numpy(np.concatenate([x.v_prefix, x.v_suffix[off[g]:off[g + 1]]])).double()
        q_full = torch.zeros(P + S, 6, 16, dtype=torch.float64)
        q_full[P:] = torch.from_numpy(x.q[off[g]:off[g + 1]]).double()
        kk = k_full.repeat_interleave(r, dim=1).permute(1, 0, 2)[None]   # [1,Hq,L,D]
        vv = v_full.repeat_interleave(r, dim=1).permute(1, 0, 2)[None]
        qq = q_full.permute(1, 0, 2)[None]
        o = torch.nn.functional.scaled_dot_product_attention(qq, kk, vv, is_causal=True, scale=scale)
        o = o[0].permute(1, 0, 2).numpy()[P:]
        assert np.abs(o - out[off[g]:off[g + 1]]).max() < 1e-12
        # LSE via torch.logsumexp of the masked scores
        sc = scale * torch.einsum("hid,hjd->hij", qq[0], kk[0])
        mask = torch.ones(P + S, P + S, dtype=torch.bool).tril()
        l = torch.logsumexp(sc.masked_fill(~mask, float("-inf")), dim=-1).numpy()[:, P:]
        assert np.abs(l - lse[:, off[g]:off[g + 1]]).max() < 1e-12


# ---- P6: rollouts are isolated from each other
@pytest.mark.parametrize("run", IMPLS)
def test_p6_rollout_isolation(run):
    x = tiny(seed=5, lens=(4, 3, 5))
    out0, lse0 = run(x)
    off = ref.suffix_offsets(x.suffix_lens)
    sl = slice(off[1], off[2])
    for a in (x.q, x.k_suffix, x.v_suffix):
        a[sl] = a[sl] * 2 + 1
    out1, lse1 = run(x)
    for g in (0, 2):
        keep = slice(off[g], off[g + 1])
        assert np.array_equal(out0[keep], out1[keep])
        assert np.array_equal(lse0[:, keep], lse1[:, keep])
    assert not np.array_equal(out0[sl], out1[sl])


# ---- P7: the prefix rectangle has no order
@pytest.mark.parametrize("run", IMPLS)
def test_p7_prefix_permutation(run):
    x = tiny(seed=6, P=11)
    out0, lse0 = run(x)
    perm = np.random.default_rng(1).permutation(11)
    x.k_prefix = np.ascontiguousarray(x.k_prefix[perm])
    x.v_prefix = np.ascontiguousarray(x.v_prefix[perm])
    out1, lse1 = run(x)
    assert np.abs(out0 - out1).max() < 1e-13
    assert np.abs(lse0 - lse1).max() < 1e-13


# ---- P8: a vector common to all keys of a head shifts LSE by scale*<q,mu>, leaves O unchanged
@pytest.mark.parametrize("run", IMPLS)
def test_p8_key_shift(run):
    x = tiny(seed=7, dtype="bf16")   # bf16-valued keys + a coarse-grid shift add exactly in fp32
    scale = 0.41
    out0, lse0 = run(x, scale)
    mu = (np.round(np.random.default_rng(2).standard_normal((2, 8)) * 8) / 16).astype(np.float32)
    x.k_prefix = x.k_prefix + mu[None]
    x.k_suffix = x.k_suffix + mu[None]
    out1, lse1 = run(x, scale)
    assert np.abs(out0 - out1).max() < 1e-12
    for h in range(4):
        shift = scale * (x.q[:, h].astype(np.float64) @ mu[h // 2].astype(np.float64))
        assert np.abs(lse1[h] - lse0[h] - shift).max() < 1e-12


# ---- P9: split/merge identity for arbitrary splits, associativity, empty side
def test_p9_split_merge_identity():
    rng = np.random.default_rng(8)
    M, N, D = 5, 13, 6
    q, k, v = rng.standard_normal((M, D)), rng.standard_normal((N, D)), rng.standard_normal((N, D))
    o_all, l_all = ref.partial_attention(q, k, v, 0.5)
    for cut in (0, 1, 6, 12, 13):
        oa, la = ref.partial_attention(q, k[:cut], v[:cut], 0.5)
        ob, lb = ref.partial_attention(q, k[cut:], v[cut:], 0.5)
        o, l = ref.merge_partials(oa, la, ob, lb)
        assert np.abs(o - o_all).max() < 1e-13 and np.abs(l - l_all).max() < 1e-13
    idx = rng.permutation(N)
    A, B, C = idx[:4], idx[4:9], idx[9:]
    pa, pb, pc = (ref.partial_attention(q, k[s], v[s], 0.5) for s in (A, B, C))
    left = ref.merge_partials(*ref.merge_partials(*pa, *pb), *pc)
    right = ref.merge_partials(*pa, *ref.merge_partials(*pb, *pc))
    for got in (left, right):
        assert np.abs(got[0] - o_all).max() < 1e-13 and np.abs(got[1] - l_all).max() < 1e-13
    # both sides empty stays empty, no NaN
    o, l = ref.merge_partials(np.zeros((2, 3)), np.full(2, -np.inf), np.zeros((2, 3)), np.full(2, -np.inf))
    assert (o == 0).all() and np.isneginf(l).all()


def test_p9_prefix_suffix_split_is_the_oracle():
    """The exact split the three kernels use: prefix partial (+) causal suffix partial."""
    x = tiny(seed=10, P=7, lens=(4, 2))
    scale = 0.3
    out, lse = run_np(x, scale)
    off = ref.suffix_offsets(x.suffix_lens)
    for g, S in enumerate(x.suffix_lens):
        for h in range(4):
            c = h // 2
            for i in range(S):
                t = off[g] + i
                p1 = ref.partial_attention(x.q[t:t + 1, h], x.k_prefix[:, c], x.v_prefix[:, c], scale)
                p2 = ref.partial_attention(x.q[t:t + 1, h], x.k_suffix[off[g]:t + 1, c], x.v_suffix[off[g]:t + 1, c], scale)
                o, l = ref.merge_partials(*p1, *p2)
                assert np.abs(o[0] - out[t, h]).max() < 1e-13 and abs(l[0] - lse[h, t]) < 1e-13


# ---- P10: a single visible key
@pytest.mark.parametrize("run", IMPLS)
def test_p10_single_key(run):
    x = tiny(seed=11, P=0, lens=(1, 1))
    scale = 0.77
    out, lse = run(x, scale)
    for t in range(2):
        for h in range(4):
            c = h // 2
            assert np.array_equal(out[t, h], x.v_suffix[t, c].astype(np.float64))
            want = scale * float(x.q[t, h].astype(np.float64) @ x.k_suffix[t, c].astype(np.float64))
            assert abs(lse[h, t] - want) < 1e-14


# ---- P11: one dominating key
@pytest.mark.parametrize("run", IMPLS)
def test_p11_peaked_row(run):
    x = tiny(seed=12, Hq=1, Hkv=1, D=8, P=9, lens=(2,))
    x.q[...] = 0
    x.q[:, 0, 0] = 1.0
    x.k_prefix[...] = 0
    x.k_suffix[...] = 0
    x.k_prefix[4, 0, 0] = 200.0
    out, lse = run(x, 1.0)
    for t in range(2):
        assert np.abs(out[t, 0] - x.v_prefix[4, 0]).max() < 1e-12
        assert abs(lse[0, t] - 200.0) < 1e-12


# ---- P12: GQA mapping h -> h // r
@pytest.mark.parametrize("run", IMPLS)
def test_p12_gqa_equals_repeated_kv(run):
    x = tiny(seed=13, Hq=6, Hkv=3, D=8, P=4, lens=(3, 2))
    out, lse = run(x)
    y = tiny(seed=13, Hq=6, Hkv=3, D=8, P=4, lens=(3, 2))
    y.k_prefix, y.v_prefix, y.k_suffix, y.v_suffix = (np.ascontiguousarray(np.repeat(a, 2, axis=1))
                                                      for a in (x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix))
    out2, lse2 = run(y)   # now Hq == Hkv: plain multi-head attention
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)
    # distinct V per kv head means a wrong mapping would be visible
    assert not np.allclose(out[:, 0], out[:, 2])


# ---- hand-worked example with typed-in expected values
@pytest.mark.parametrize("run", IMPLS)
def test_hand_worked_golden(run):
    with open(os.path.join(GOLDEN, "hand_worked.json")) as f:
        gold = json.load(f)
    for case in gold["cases"]:
        a = {k: np.asarray(case[k], dtype=np.float32) for k in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")}
        x = wl.Inputs(wl.Workload("gold", "f32", a["q"].shape[1], a["k_suffix"].shape[1], a["q"].shape[2],
                                  a["k_prefix"].shape[0], 1, 0, len(case["suffix_lens"]), None),
                      np.asarray(case["suffix_lens"], np.int32), a["q"], a["k_prefix"], a["v_prefix"], a["k_suffix"], a["v_suffix"])
        out, lse = run(x, case["scale"])
        assert np.abs(out - np.asarray(case["out"])).max() < 1e-12, case["name"]
        want = np.array([[math.log(v) for v in row] for row in case["exp_lse"]])
        assert np.abs(lse - want).max() < 1e-12, case["name"]


# ---- the two oracle versions agree with each other on a ragged multi-tile case, full and by rows
def test_c_oracle_equals_numpy_definition():
    x = wl.make_custom("bf16", 14, 2, 32, 70, (33, 1, 18), seed=21)
    o_np, l_np = run_np(x)
    o_c, l_c = run_c(x)
    assert np.abs(o_np - o_c).max() < 1e-12 and np.abs(l_np - l_c).max() < 1e-12
    rows = np.array([0, 32, 33, 34, 51], dtype=np.int64)
    o_r, l_r = run_c(x, rows=rows)
    assert np.abs(o_r - o_np[rows]).max() < 1e-12 and np.abs(l_r - l_np[:, rows]).max() < 1e-12
    o_r2, l_r2 = ref.prefix_shared_attention_rows(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                  x.suffix_lens, x.workload.scale, rows)
    assert np.abs(o_r2 - o_np[rows]).max() < 1e-12 and np.abs(l_r2 - l_np[:, rows]).max() < 1e-12


def test_planted_mistakes_are_caught():
    """A wrong diagonal (exclusive) or a swapped K/V would fail P4's brute force: plant them in a copy."""
    x = tiny(seed=3, Hq=1, Hkv=1, D=4, P=2, lens=(3,))
    out, lse = run_np(x, 0.5)
    k_full = np.concatenate([x.k_prefix[:, 0], x.k_suffix[:, 0]])
    v_full = np.concatenate([x.v_prefix[:, 0], x.v_suffix[:, 0]])
    q_full = np.concatenate([np.zeros((2, 4)), x.q[:, 0]])
    o_ok, _ = ref.full_causal_attention_bruteforce(q_full, k_full, v_full, 0.5)
    assert np.abs(o_ok[2:] - out[:, 0]).max() < 1e-12
    o_swapped, _ = ref.full_causal_attention_bruteforce(q_full, v_full, k_full, 0.5)
    assert np.abs(o_swapped[2:] - out[:, 0]).max() > 1e-3
