"""Pins for the log-probability / advantage oracle, CPU only."""
import math

import numpy as np
import pytest

from oracle import ref_logprob as ref


def tiny(seed=0, N=5, d=6, V=11):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((N, d)), rng.standard_normal((V, d)), rng.integers(0, V, size=N)


def test_l1_zero_head_gives_uniform_distribution():
    h, w, y = tiny()
    lp, lse = ref.token_logprobs(h, np.zeros_like(w), y)
    assert np.abs(lp + math.log(11)).max() < 1e-14 and np.abs(lse - math.log(11)).max() < 1e-14


def test_l2_one_hot_logits_closed_form():
    # orthogonal head rows: z_v = a * h[v]; with h = e_k * t the logits are t at v = k and 0 elsewhere
    V = d = 7
    w = np.eye(V)
    t = 3.5
    h = np.zeros((2, d))
    h[0, 2] = t
    h[1, 5] = t
    lp, lse = ref.token_logprobs(h, w, np.array([2, 0]))
    z = math.log(math.exp(t) + (V - 1))
    assert abs(lse[0] - z) < 1e-14 and abs(lp[0] - (t - z)) < 1e-14
    assert abs(lp[1] - (0.0 - z)) < 1e-14


def test_l3_matches_bruteforce_loops():
    h, w, y = tiny(seed=1)
    lp, _ = ref.token_logprobs(h, w, y, logit_scale=0.7)
    assert np.abs(lp - ref.token_logprobs_bruteforce(h, w, y, 0.7)).max() < 1e-13


def test_l4_matches_torch_log_softmax_gather():
    import torch
    h, w, y = tiny(seed=2, N=9, d=16, V=50)
    lp, lse = ref.token_logprobs(h, w, y, logit_scale=1.3, chunk=4)
    z = 1.3 * torch.tensor(h) @ torch.tensor(w).T
    want = torch.log_softmax(z, dim=1).gather(1, torch.tensor(y)[:, None])[:, 0].numpy()
    assert np.abs(lp - want).max() < 1e-12
    assert np.abs(lse - torch.logsumexp(z, dim=1).numpy()).max() < 1e-12


def test_l5_probabilities_over_all_targets_sum_to_one():
    h, w, _ = tiny(seed=3, N=3, d=5, V=13)
    tot = np.zeros(3)
    for v in range(13):
        lp, _ = ref.token_logprobs(h, w, np.full(3, v))
        tot += np.exp(lp)
    assert np.abs(tot - 1).max() < 1e-13


def test_l6_logit_shift_and_temperature():
    h, w, y = tiny(seed=4)
    lp, lse = ref.token_logprobs(h, w, y)
    u = np.linspace(-1, 1, 6)
    lp2, lse2 = ref.token_logprobs(h, w + u, y)        # every logit of token n moves by <u, h_n>
    assert np.abs(lp2 - lp).max() < 1e-12
    assert np.abs((lse2 - lse) - h @ u).max() < 1e-12
    lp3, _ = ref.token_logprobs(h, w, y, logit_scale=0.5)
    lp4, _ = ref.token_logprobs(0.5 * h, w, y)
    assert np.abs(lp3 - lp4).max() < 1e-13


def test_l7_planted_mistakes_are_caught():
    h, w, y = tiny(seed=5)
    good, lse = ref.token_logprobs(h, w, y)
    brute = ref.token_logprobs_bruteforce(h, w, y)
    z = h @ w.T
    wrong_gather = z[np.arange(5), (y + 1) % 11] - lse                 # off-by-one target
    no_max = z[np.arange(5), y] - np.log(np.exp(z).sum(1)) + 1e-3      # dropped/extra term
    transposed = (w @ h.T)[y, np.arange(5)] - np.log(np.exp(z.T).sum(1))[y]   # normalised over tokens instead of vocabulary
    for bad in (wrong_gather, no_max, transposed):
        assert np.abs(bad - brute).max() > 1e-4
    assert np.abs(good - brute).max() < 1e-13


def test_a1_advantages_hand_worked_and_invariants():
    a = ref.group_advantages([1.0, 0.0, 0.0, 1.0])
    assert np.allclose(a, [1, -1, -1, 1])
    a = ref.group_advantages([2.0, 0.0, 0.0, 0.0])                    # mean 0.5, population std sqrt(0.75)
    assert np.allclose(a, np.array([1.5, -0.5, -0.5, -0.5]) / math.sqrt(0.75))
    r = np.array([0.3, 1.0, 0.0, 0.7, 0.7, 0.1, 1.0, 0.2])
    a = ref.group_advantages(r)
    assert abs(a.mean()) < 1e-15 and abs((a ** 2).mean() - 1) < 1e-14
    assert np.allclose(ref.group_advantages(3 * r + 5), a)            # affine rescaling of rewards changes nothing
    assert np.allclose(ref.group_advantages(-r), -a)
    assert (ref.group_advantages([0.5] * 8) == 0).all()               # no signal in a group of equal rewards


def test_hand_worked_logprob_golden():
    import json
    import os
    cases = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked_backward_logprob.json")))["logprob_cases"]
    for c in cases:
        lp, lse = ref.token_logprobs(np.array(c["hidden"]), np.array(c["lm_head"]), np.array(c["targets"]), c["logit_scale"])
        assert np.abs(lp - np.array(c["logprob"])).max() < 1e-14, c["name"]
        assert np.abs(lse - np.array(c["lse"])).max() < 1e-14, c["name"]
