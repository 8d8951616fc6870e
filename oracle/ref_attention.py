"""fp64 CPU oracle for prefix-shared GRPO prefill attention.  TEST INFRASTRUCTURE ONLY.

This module is the definition the HIP path is checked against.  It is imported
only by tests, by the smoke check and by the benchmark's cpu_baseline leg; the
product path never calls it and shares no code with it.

What is computed (paper Sec. 5.1: the gathered video embeddings are encoded once
and reused by every rollout of a step; Sec. 5.2: every rollout is prefilled over
the whole multimodal sequence by the policy and the reference model; Sec. 4.2 /
Eq. 1: G responses o_1..o_G are sampled for one question):

  For rollout g, query head h (kv head c = h // (Hq // Hkv)) and suffix row i the
  visible keys are the P shared prefix tokens and the rollout's own suffix tokens
  0..i (inclusive diagonal).  With s_j = scale * <q, k_j>:

      m   = max_j s_j
      Z   = sum_j exp(s_j - m)
      LSE = m + ln Z
      O   = sum_j exp(s_j - m) / Z * v_j

  i.e. ordinary causal softmax attention of the sequence
  [video prefix | prompt | response_g], restricted to its last S_g rows.

Everything is float64, softmax is two-pass, there is no tiling, no online
rescaling and no merge of partial results in `prefix_shared_attention`.

Pins (tests/test_oracle_pins.py): row sums, uniform-score closed form, causality,
equality with brute-force full-sequence attention, torch SDPA on the concatenated
sequence, rollout isolation, prefix permutation, key shift, split/merge identity,
single key, peaked row, GQA-vs-repeated-KV.  The backward (bottom of this file) is
pinned by finite differences of the forward, torch autograd, closed forms and invariants.
"""
from __future__ import annotations

import numpy as np


def _as64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def suffix_offsets(suffix_lens):
    """off_g = sum of S_g' for g' < g; returns array of G+1 offsets (last = T)."""
    lens = np.asarray(suffix_lens, dtype=np.int64)
    off = np.zeros(len(lens) + 1, dtype=np.int64)
    off[1:] = np.cumsum(lens)
    return off


def visible_scores(q, k_prefix, k_suffix, suffix_lens, scale, g, h):
    """Scaled scores of rollout g, q-head h against its visible keys.

    Returns (scores [S_g, P + S_g] with -inf at masked positions, c = kv head).
    Column j < P is prefix token j; column P + j' is the rollout's suffix token j'.
    """
    q, k_prefix, k_suffix = _as64(q), _as64(k_prefix), _as64(k_suffix)
    T, Hq, D = q.shape
    P, Hkv, _ = k_prefix.shape
    off = suffix_offsets(suffix_lens)
    r = Hq // Hkv
    c = h // r
    S = int(off[g + 1] - off[g])
    qg = q[off[g]:off[g + 1], h, :]                       # [S, D]
    keys = np.concatenate([k_prefix[:, c, :], k_suffix[off[g]:off[g + 1], c, :]], axis=0)  # [P+S, D]
    s = scale * (qg @ keys.T)                             # [S, P+S]
    i = np.arange(S)[:, None]
    j = np.arange(S)[None, :]
    s[:, P:][j > i] = -np.inf                             # causal inside the suffix, diagonal visible
    return s, c


def attention_weights(q, k_prefix, k_suffix, suffix_lens, scale, g, h):
    """Softmax weights [S_g, P + S_g] and LSE [S_g] for (rollout g, head h)."""
    s, _ = visible_scores(q, k_prefix, k_suffix, suffix_lens, scale, g, h)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    Z = e.sum(axis=1, keepdims=True)
    return e / Z, (m + np.log(Z))[:, 0]


def prefix_shared_attention(q, k_prefix, v_prefix, k_suffix, v_suffix, suffix_lens, scale):
    """The definition above for every (g, h, i).

    q [T,Hq,D]; k_prefix, v_prefix [P,Hkv,D]; k_suffix, v_suffix [T,Hkv,D];
    suffix_lens [G] with sum T.  Returns out [T,Hq,D] float64, lse [Hq,T] float64.
    """
    q, v_prefix, v_suffix = _as64(q), _as64(v_prefix), _as64(v_suffix)
    T, Hq, D = q.shape
    off = suffix_offsets(suffix_lens)
    assert off[-1] == T, "suffix_lens must sum to T"
    out = np.zeros((T, Hq, D), dtype=np.float64)
    lse = np.zeros((Hq, T), dtype=np.float64)
    for g in range(len(suffix_lens)):
        for h in range(Hq):
            w, l = attention_weights(q, k_prefix, k_suffix, suffix_lens, scale, g, h)
            c = h // (Hq // v_prefix.shape[1])
            vals = np.concatenate([v_prefix[:, c, :], v_suffix[off[g]:off[g + 1], c, :]], axis=0)
            out[off[g]:off[g + 1], h, :] = w @ vals
            lse[h, off[g]:off[g + 1]] = l
    return out, lse


def prefix_shared_attention_rows(q, k_prefix, v_prefix, k_suffix, v_suffix, suffix_lens, scale, rows):
    """Same definition, only for the packed token rows listed in `rows` (all heads).

    Returns out [len(rows),Hq,D], lse [Hq,len(rows)].  Used where the full tensor is
    too large for the CPU; each row is computed one by one against its full key set.
    """
    T, Hq, D = q.shape
    P, Hkv, _ = k_prefix.shape
    off = suffix_offsets(suffix_lens)
    r = Hq // Hkv
    rows = np.asarray(rows, dtype=np.int64)
    out = np.zeros((len(rows), Hq, D), dtype=np.float64)
    lse = np.zeros((Hq, len(rows)), dtype=np.float64)
    for n, t in enumerate(rows):
        g = int(np.searchsorted(off, t, side="right") - 1)
        i = int(t - off[g])
        for c in range(Hkv):
            keys = np.concatenate([_as64(k_prefix[:, c, :]), _as64(k_suffix[off[g]:off[g] + i + 1, c, :])], axis=0)
            vals = np.concatenate([_as64(v_prefix[:, c, :]), _as64(v_suffix[off[g]:off[g] + i + 1, c, :])], axis=0)
            for h in range(c * r, (c + 1) * r):
                s = scale * (keys @ _as64(q[t, h, :]))
                m = s.max()
                e = np.exp(s - m)
                Z = e.sum()
                out[n, h, :] = (e / Z) @ vals
                lse[h, n] = m + np.log(Z)
    return out, lse


def full_causal_attention_bruteforce(q, k, v, scale):
    """Textbook single-head causal attention with explicit Python loops.

    q, k, v [L, D].  Row i sees keys 0..i.  Deliberately written without matmul,
    masks or broadcasting so that it shares nothing with the functions above.
    Returns out [L, D], lse [L].
    """
    L, D = len(q), len(q[0])
    out = [[0.0] * D for _ in range(L)]
    lse = [0.0] * L
    for i in range(L):
        s = []
        for j in range(i + 1):
            acc = 0.0
            for d in range(D):
                acc += float(q[i][d]) * float(k[j][d])
            s.append(scale * acc)
        m = max(s)
        e = [float(np.exp(x - m)) for x in s]
        Z = sum(e)
        for j in range(i + 1):
            wj = e[j] / Z
            for d in range(D):
                out[i][d] += wj * float(v[j][d])
        lse[i] = m + float(np.log(Z))
    return np.array(out), np.array(lse)


def partial_attention(q_rows, keys, vals, scale):
    """Attention of query rows [M, D] over an explicit key/value set [N, D], no mask.

    Returns (O [M, D], LSE [M]); an empty key set gives (0, -inf).  This is the
    'partial result' that the prefix pass and the suffix pass each produce.
    """
    q_rows, keys, vals = _as64(q_rows), _as64(keys), _as64(vals)
    M, D = q_rows.shape
    if keys.shape[0] == 0:
        return np.zeros((M, D)), np.full((M,), -np.inf)
    s = scale * (q_rows @ keys.T)
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    Z = e.sum(axis=1, keepdims=True)
    return (e / Z) @ vals, (m + np.log(Z))[:, 0]


def merge_partials(o1, lse1, o2, lse2):
    """Combine two normalised partial results over disjoint key sets.

    LSE = ln(e^{LSE1} + e^{LSE2});  O = e^{LSE1-LSE} O1 + e^{LSE2-LSE} O2.
    A side with LSE = -inf (no keys) contributes nothing.  o* [M, D], lse* [M].
    """
    o1, o2, lse1, lse2 = _as64(o1), _as64(o2), _as64(lse1), _as64(lse2)
    m = np.maximum(lse1, lse2)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w1 = np.exp(lse1 - m_safe)
    w2 = np.exp(lse2 - m_safe)
    tot = w1 + w2
    with np.errstate(invalid="ignore", divide="ignore"):
        lse = np.where(np.isfinite(m), m_safe + np.log(tot), -np.inf)
        a1 = np.where(tot > 0, w1 / tot, 0.0)
        a2 = np.where(tot > 0, w2 / tot, 0.0)
    return a1[:, None] * o1 + a2[:, None] * o2, lse


# ----------------------------------------------------------------------------------------------
# Backward.  The policy model is trained through the attention (paper Eq. 1 is maximised by
# gradient ascent on the policy's token probabilities; Sec. 5.2 prefills every rollout with the
# policy model), so the gradient of a scalar objective L with respect to the attention inputs is
# needed, given dO = dL/dO.  What follows is the chain rule applied to the forward definition
# at the top of this file, one (rollout, head) at a time, in fp64:
#
#     W   = softmax(s) over the visible keys            (row-wise; `attention_weights`)
#     dV  = W^T dO
#     dW  = dO V^T
#     dS  = W * (dW - rowsum(W * dW))                   (Jacobian of a row-wise softmax)
#     dQ  = scale * dS K,      dK = scale * dS^T Q
#
# A kv head receives the sum over the q heads of its group; a *prefix* key/value additionally
# receives the sum over all G rollouts, because every rollout attends to the same cached prefix
# (Sec. 5.1).  The LSE output is treated as a saved statistic, not as a differentiated output.
# Pinned against central finite differences of `prefix_shared_attention`, torch autograd on the
# concatenated sequences, closed forms and invariants (tests/test_oracle_pins.py).

def prefix_shared_attention_backward(q, k_prefix, v_prefix, k_suffix, v_suffix, suffix_lens, scale, d_out):
    """Gradients of L = sum(d_out * out) with respect to the five inputs.

    d_out [T,Hq,D].  Returns (dq [T,Hq,D], dk_prefix [P,Hkv,D], dv_prefix [P,Hkv,D],
    dk_suffix [T,Hkv,D], dv_suffix [T,Hkv,D]), all float64.
    """
    q, k_prefix, v_prefix = _as64(q), _as64(k_prefix), _as64(v_prefix)
    k_suffix, v_suffix, d_out = _as64(k_suffix), _as64(v_suffix), _as64(d_out)
    T, Hq, D = q.shape
    P, Hkv, _ = k_prefix.shape
    r = Hq // Hkv
    off = suffix_offsets(suffix_lens)
    dq = np.zeros_like(q)
    dkp, dvp = np.zeros_like(k_prefix), np.zeros_like(v_prefix)
    dks, dvs = np.zeros_like(k_suffix), np.zeros_like(v_suffix)
    for g in range(len(suffix_lens)):
        a, b = int(off[g]), int(off[g + 1])
        for h in range(Hq):
            c = h // r
            w, _ = attention_weights(q, k_prefix, k_suffix, suffix_lens, scale, g, h)   # [S, P+S]
            keys = np.concatenate([k_prefix[:, c, :], k_suffix[a:b, c, :]], axis=0)
            vals = np.concatenate([v_prefix[:, c, :], v_suffix[a:b, c, :]], axis=0)
            do = d_out[a:b, h, :]
            dvals = w.T @ do
            dw = do @ vals.T
            ds = w * (dw - (w * dw).sum(axis=1, keepdims=True))
            dq[a:b, h, :] = scale * (ds @ keys)
            dkeys = scale * (ds.T @ q[a:b, h, :])
            dkp[:, c, :] += dkeys[:P]
            dvp[:, c, :] += dvals[:P]
            dks[a:b, c, :] += dkeys[P:]
            dvs[a:b, c, :] += dvals[P:]
    return dq, dkp, dvp, dks, dvs
