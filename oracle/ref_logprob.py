"""fp64 CPU oracle for response-token log-probabilities and group advantages.  TEST INFRASTRUCTURE ONLY.

Imported only by tests, the smoke check and the benchmark's cpu_baseline leg; the product path
never calls it and shares no code with it.

What is computed.  The GRPO objective (paper Eq. 1) is built from the probabilities that the
policy, the old policy and the reference model assign to the sampled responses; after the
prefill every device computes the logits of its token slice (Sec. 5.2).  For token n with
final hidden state h_n, LM-head matrix W [V, d] and sampled token id y_n:

    z_v      = logit_scale * <w_v, h_n>            (logit_scale = 1 / sampling temperature)
    LSE_n    = ln sum_v exp(z_v)
    logp_n   = z_{y_n} - LSE_n                      = ln softmax(z)[y_n]

Two-pass (max, then sum) in float64; the matrix product is a library step (numpy matmul),
taken in token chunks only to bound memory.

Eq. 2: rewards r_1..r_G of the G responses to one question are normalised to advantages
A_i = (r_i - mean(r)) / std(r).  Reading where the paper is silent: std is the population
standard deviation of the G rewards (divide by G); a group whose rewards are all equal carries
no signal and gets A_i = 0.

Pins (tests/test_oracle_logprob_pins.py): closed forms (zero LM head, one-hot logits), a
loop-only brute force, torch log_softmax + gather, normalisation over all targets, logit-shift
invariance, temperature as a rescaling of h; advantages: zero mean / unit variance, affine
invariance, hand-worked values.
"""
from __future__ import annotations

import numpy as np


def token_logprobs(hidden, lm_head, targets, logit_scale=1.0, chunk=256):
    """hidden [N, d], lm_head [V, d], targets [N] int.  Returns (logp [N], lse [N]) float64."""
    h = np.asarray(hidden, dtype=np.float64)
    w = np.asarray(lm_head, dtype=np.float64)
    y = np.asarray(targets, dtype=np.int64)
    N, V = h.shape[0], w.shape[0]
    assert h.shape[1] == w.shape[1] and y.shape == (N,)
    assert ((y >= 0) & (y < V)).all(), "target id out of range"
    logp = np.empty(N, dtype=np.float64)
    lse = np.empty(N, dtype=np.float64)
    for a in range(0, N, chunk):
        z = float(logit_scale) * (h[a:a + chunk] @ w.T)          # [n, V]
        m = z.max(axis=1)
        l = m + np.log(np.exp(z - m[:, None]).sum(axis=1))
        lse[a:a + chunk] = l
        logp[a:a + chunk] = z[np.arange(z.shape[0]), y[a:a + chunk]] - l
    return logp, lse


def token_logprobs_bruteforce(hidden, lm_head, targets, logit_scale=1.0):
    """The same definition with explicit Python loops (tiny inputs only); shares nothing with the above."""
    N, d, V = len(hidden), len(hidden[0]), len(lm_head)
    out = []
    for n in range(N):
        z = []
        for v in range(V):
            acc = 0.0
            for k in range(d):
                acc += float(hidden[n][k]) * float(lm_head[v][k])
            z.append(logit_scale * acc)
        m = max(z)
        s = sum(float(np.exp(x - m)) for x in z)
        out.append(z[int(targets[n])] - (m + float(np.log(s))))
    return np.array(out)


def group_advantages(rewards):
    """Eq. 2 for one group of G rewards; population std; all-equal rewards give zeros."""
    r = np.asarray(rewards, dtype=np.float64)
    mean = r.mean()
    std = np.sqrt(((r - mean) ** 2).mean())
    if std == 0.0:
        return np.zeros_like(r)
    return (r - mean) / std
