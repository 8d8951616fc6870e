"""Seeded synthetic workloads: shapes, value distributions and byte/FLOP accounting.

Holds none of the attention arithmetic.  Both the HIP path's tests/benchmark and
the CPU oracle's tests draw their inputs from here, so the two sides consume
bit-identical values.

Shapes follow the paper's long-video RL workloads: 512 frames (the frame count of
its efficiency comparison and Video-MME evaluation, Sec. 6), 3,600 frames
(hour-long videos, Sec. 1 / Sec. 7) and 8,192 frames (maximum, Sec. 1), a 7B
decoder (28 query heads, 4 kv heads, head_dim 128), G = 8..16 rollouts per
question (Sec. 4.2, Sec. 5.1) and batch size 1 per GPU (Sec. 6.2).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16"
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    frames: int
    tokens_per_frame: int
    prompt_len: int
    num_rollouts: int
    response_len: Optional[int]            # fixed response length, or None when ragged
    response_range: Optional[tuple] = None  # inclusive (lo, hi) when ragged
    key_offset: Optional[str] = None        # None | "all" (every key) | "prefix" (video keys only)
    key_offset_std: float = 0.5
    seed: int = 0
    note: str = ""

    @property
    def prefix_len(self) -> int:
        return self.frames * self.tokens_per_frame

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.head_dim))


WORKLOADS = {
    "C1": Workload("C1", "f32", 1, 1, 64, 16, 16, 32, 2, 64, note="tiny fp32, full-tensor parity"),
    "C2": Workload("C2", "bf16", 28, 4, 128, 64, 64, 128, 8, 1024, note="one 7B-shaped layer, 4K prefix"),
    "C3": Workload("C3", "bf16", 28, 4, 128, 512, 64, 256, 8, 2048, key_offset="all",
                   note="512 frames, 32K prefix, per-head key mean offset; the graded configuration"),
    "C3pre": Workload("C3pre", "bf16", 28, 4, 128, 512, 64, 256, 8, 2048, key_offset="prefix",
                      note="C3 shape with the key offset on video keys only (moves mass between the partials)"),
    "C4": Workload("C4", "bf16", 28, 4, 128, 3600, 64, 256, 8, 2048, note="hour-long video, 230K prefix"),
    "C5": Workload("C5", "bf16", 28, 4, 128, 8192, 64, 512, 16, None, response_range=(256, 4096),
                   note="max frames, 512K prefix, ragged rollouts"),
    # The other half of "computed once": causal self-attention of the 512-frame video prefix itself
    # (P = 0, one sequence of 32,768 video tokens), run once per layer and shared by all rollouts.
    "N1": Workload("N1", "bf16", 28, 4, 128, 0, 64, 0, 1, 32768,
                   note="shared prefix self-attention: 32K video tokens, causal, no rollouts"),
    # the same for the hour-long video of C4: 3,600 frames x 64 tokens in one causal sequence
    "N1h": Workload("N1h", "bf16", 28, 4, 128, 0, 64, 0, 1, 230400,
                    note="shared prefix self-attention of an hour-long video: 230,400 tokens, causal"),
}


def round_to_bf16(x: np.ndarray):
    """Round fp32 to bf16 (round-to-nearest-even).  Returns (uint16 bit patterns, fp32 widened values)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    rounded = (bits + np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    u16 = rounded.astype(np.uint16)
    widened = (u16.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return u16, widened


def draw_suffix_lens(w: Workload, rng) -> np.ndarray:
    if w.response_len is not None:
        resp = np.full(w.num_rollouts, w.response_len, dtype=np.int64)
    else:
        lo, hi = w.response_range
        resp = rng.integers(lo, hi + 1, size=w.num_rollouts)
    return (w.prompt_len + resp).astype(np.int32)


@dataclass
class Inputs:
    workload: Workload
    suffix_lens: np.ndarray            # int32 [G]
    # exact values both sides consume, as fp32 (bf16 workloads: already rounded)
    q: np.ndarray
    k_prefix: np.ndarray
    v_prefix: np.ndarray
    k_suffix: np.ndarray
    v_suffix: np.ndarray
    bits: dict = field(default_factory=dict)   # bf16 workloads: name -> uint16 bit patterns

    @property
    def total_suffix(self) -> int:
        return int(self.suffix_lens.sum())


def make_inputs(w: Workload, seed: Optional[int] = None, keep_f32: bool = True) -> Inputs:
    """Draw order is fixed: lengths, q, k_prefix, v_prefix, k_suffix, v_suffix, key offsets."""
    rng = np.random.default_rng(w.seed if seed is None else seed)
    lens = draw_suffix_lens(w, rng)
    T, P = int(lens.sum()), w.prefix_len
    shapes = {
        "q": (T, w.num_q_heads, w.head_dim),
        "k_prefix": (P, w.num_kv_heads, w.head_dim),
        "v_prefix": (P, w.num_kv_heads, w.head_dim),
        "k_suffix": (T, w.num_kv_heads, w.head_dim),
        "v_suffix": (T, w.num_kv_heads, w.head_dim),
    }
    raw = {n: rng.standard_normal(s, dtype=np.float32) for n, s in shapes.items()}
    if w.key_offset is not None:
        mu = (w.key_offset_std * rng.standard_normal((w.num_kv_heads, w.head_dim))).astype(np.float32)
        raw["k_prefix"] += mu[None]
        if w.key_offset == "all":
            raw["k_suffix"] += mu[None]
    vals, bits = {}, {}
    for n, a in raw.items():
        if w.dtype == "bf16":
            b, wd = round_to_bf16(a)
            bits[n] = b
            vals[n] = wd if keep_f32 else None
        else:
            vals[n] = a
    return Inputs(w, lens, vals["q"], vals["k_prefix"], vals["v_prefix"], vals["k_suffix"],
                  vals["v_suffix"], bits)


def make_custom(dtype, Hq, Hkv, D, P, suffix_lens, seed=0, name="custom", std=1.0) -> Inputs:
    """Inputs for an arbitrary shape (edge-case tests); iid N(0, std^2)."""
    rng = np.random.default_rng(seed)
    lens = np.asarray(suffix_lens, dtype=np.int32)
    T = int(lens.sum())
    w = Workload(name, dtype, Hq, Hkv, D, P, 1, 0, len(lens), None, seed=seed)
    raw = {
        "q": rng.standard_normal((T, Hq, D), dtype=np.float32) * np.float32(std),
        "k_prefix": rng.standard_normal((P, Hkv, D), dtype=np.float32) * np.float32(std),
        "v_prefix": rng.standard_normal((P, Hkv, D), dtype=np.float32),
        "k_suffix": rng.standard_normal((T, Hkv, D), dtype=np.float32) * np.float32(std),
        "v_suffix": rng.standard_normal((T, Hkv, D), dtype=np.float32),
    }
    vals, bits = {}, {}
    for n, a in raw.items():
        if dtype == "bf16":
            bits[n], vals[n] = round_to_bf16(a)
        else:
            vals[n] = a
    return Inputs(w, lens, vals["q"], vals["k_prefix"], vals["v_prefix"], vals["k_suffix"],
                  vals["v_suffix"], bits)


_TENSORS = ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")


def _rebuild(x: Inputs, w: Workload, lens, pick) -> Inputs:
    """New Inputs whose tensors are pick(name, x's tensors), applied alike to the values and the bf16 bits."""
    src = {n: getattr(x, n) for n in _TENSORS}
    vals = {n: pick(n, src) for n in _TENSORS}
    bits = {n: pick(n, x.bits) for n in _TENSORS} if x.bits else {}
    return Inputs(w, np.asarray(lens, dtype=np.int32), vals["q"], vals["k_prefix"], vals["v_prefix"],
                  vals["k_suffix"], vals["v_suffix"], bits)


def share_prompt(x: Inputs) -> Inputs:
    """The G rollouts of a group answer the same question (Sec. 4.2), so their prompt tokens are the same
    tokens at the same positions and (the mask being causal) carry the same Q, K and V in every layer:
    copies rollout 0's prompt rows over the prompt rows of the other rollouts."""
    Lp = x.workload.prompt_len
    off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])

    def pick(name, src):
        if name.endswith("_prefix"):
            return src[name]
        b = src[name].copy()
        for g in range(1, len(x.suffix_lens)):
            b[off[g]:off[g] + Lp] = b[:Lp]
        return b
    return _rebuild(x, x.workload, x.suffix_lens, pick)


def fold_prompt(x: Inputs):
    """Two-level sharing for inputs whose prompt rows are shared (share_prompt): the prompt joins the prefix.
    Returns (prompt_call, folded_call, rows):
      prompt_call   one sequence, prefix = the video tokens, suffix = the prompt (computed once);
      folded_call   prefix = [video | prompt], suffix of rollout g = its response tokens only;
      rows          int64 [T]: for packed row t of x, the row of folded_call that holds the same token
                    (responses), or -(i + 1) for prompt token i (row i of prompt_call).
    Pure re-arrangement: no arithmetic."""
    w = x.workload
    Lp, P = w.prompt_len, w.prefix_len
    assert Lp > 0 and all(int(s) > Lp for s in x.suffix_lens)
    off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])
    resp = np.concatenate([np.arange(off[g] + Lp, off[g + 1]) for g in range(len(x.suffix_lens))])
    common = dict(dtype=w.dtype, num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                  tokens_per_frame=1, seed=w.seed)
    w_prompt = Workload(w.name + "-prompt", frames=P, prompt_len=Lp, num_rollouts=1, response_len=0, **common)
    w_folded = Workload(w.name + "-folded", frames=P + Lp, prompt_len=0, num_rollouts=w.num_rollouts,
                        response_len=None, **common)

    def pick_prompt(name, src):
        return src[name] if name.endswith("_prefix") else np.ascontiguousarray(src[name][:Lp])

    def pick_folded(name, src):
        if name.endswith("_prefix"):
            return np.concatenate([src[name], src[name[0] + "_suffix"][:Lp]])
        return np.ascontiguousarray(src[name][resp])
    prompt_call = _rebuild(x, w_prompt, [Lp], pick_prompt)
    folded_call = _rebuild(x, w_folded, x.suffix_lens - Lp, pick_folded)
    rows = np.empty(int(off[-1]), dtype=np.int64)
    rows[resp] = np.arange(len(resp))
    for g in range(len(x.suffix_lens)):
        rows[off[g]:off[g] + Lp] = -(np.arange(Lp) + 1)
    return prompt_call, folded_call, rows


def make_d_out(x: Inputs, seed: int = 1, grid: Optional[float] = None):
    """Upstream gradient dL/d(out) for the backward: iid N(0,1) of the shape of q, rounded to bf16 for
    bf16 workloads.  Returns (fp32 values both sides consume, uint16 bit patterns or None).
    With `grid` (a power of two, e.g. 1/8) the values are first rounded to multiples of it, so that
    sums of a few of them are still exact in bf16."""
    rng = np.random.default_rng(1000003 * (x.workload.seed + 1) + seed)
    raw = rng.standard_normal(x.q.shape, dtype=np.float32)
    if grid is not None:
        raw = (np.rint(raw / np.float32(grid)) * np.float32(grid)).astype(np.float32)
    if x.workload.dtype == "bf16":
        bits, vals = round_to_bf16(raw)
        return vals, bits
    return raw, None


# ---------------------------------------------------------------- response-token log-probabilities

@dataclass(frozen=True)
class LogprobWorkload:
    name: str
    num_tokens: int       # response tokens whose log-probability is needed (all rollouts of a question)
    hidden_dim: int
    vocab: int
    head_std: float = 0.02
    seed: int = 0
    note: str = ""


LOGPROB_WORKLOADS = {
    "L1": LogprobWorkload("L1", 333, 512, 5000, head_std=0.05, note="small, ragged in tokens and vocabulary"),
    "L2": LogprobWorkload("L2", 1000, 3584, 152064, note="7B-shaped LM head, 1,000 tokens"),
    # the 32K-prefix workload's responses: 8 rollouts x 2,048 response tokens, Qwen2-7B head (d = 3584, V = 152,064)
    "L3": LogprobWorkload("L3", 8 * 2048, 3584, 152064, note="8 rollouts x 2,048 response tokens, 7B-shaped LM head"),
}


@dataclass
class LogprobInputs:
    workload: LogprobWorkload
    hidden: np.ndarray      # [N, d] fp32 holding bf16-rounded values
    lm_head: np.ndarray     # [V, d] fp32 holding bf16-rounded values
    targets: np.ndarray     # [N] int32 sampled token ids
    bits: dict = field(default_factory=dict)


def make_logprob_inputs(w: LogprobWorkload, keep_f32: bool = True) -> LogprobInputs:
    """hidden ~ N(0,1) (a final-norm output), lm_head ~ N(0, head_std^2), targets uniform; all bf16-rounded.
    Draw order: hidden, lm_head, targets."""
    rng = np.random.default_rng(7919 * (w.seed + 1))
    hb, hv = round_to_bf16(rng.standard_normal((w.num_tokens, w.hidden_dim), dtype=np.float32))
    wb, wv = round_to_bf16(rng.standard_normal((w.vocab, w.hidden_dim), dtype=np.float32) * np.float32(w.head_std))
    y = rng.integers(0, w.vocab, size=w.num_tokens).astype(np.int32)
    return LogprobInputs(w, hv if keep_f32 else None, wv if keep_f32 else None, y, {"hidden": hb, "lm_head": wb})


def logprob_flop(w: LogprobWorkload) -> int:
    return 2 * w.num_tokens * w.hidden_dim * w.vocab


# ---------------------------------------------------------------- accounting (measurement only)

def visible_pairs(prefix_len: int, suffix_lens) -> int:
    """Visible (query row, key) pairs per q-head: sum_g [S_g P + S_g (S_g + 1) / 2]."""
    return int(sum(int(s) * prefix_len + int(s) * (int(s) + 1) // 2 for s in suffix_lens))


def effective_flop(Hq: int, D: int, prefix_len: int, suffix_lens) -> int:
    """4 D FLOP per visible pair (2D for QK^T, 2D for PV), all q-heads."""
    return 4 * D * Hq * visible_pairs(prefix_len, suffix_lens)


def backward_flop(Hq: int, D: int, prefix_len: int, suffix_lens) -> int:
    """10 D FLOP per visible pair: the five products S = QK^T, dW = dO V^T, dV += W^T dO, dK += dS^T Q and
    dQ += dS K, counted once each (recomputation of S and dW in the second pass is not counted)."""
    return 10 * D * Hq * visible_pairs(prefix_len, suffix_lens)


def algorithmic_bytes(w: Workload, suffix_lens) -> int:
    """Bytes the method must move at least once: Q, O, prefix K/V, suffix K/V, LSE."""
    T = int(np.sum(suffix_lens))
    e = 2 if w.dtype == "bf16" else 4
    qo = 2 * T * w.num_q_heads * w.head_dim * e
    kv = 2 * (w.prefix_len + T) * w.num_kv_heads * w.head_dim * e
    return qo + kv + 4 * w.num_q_heads * T


def sample_rows(suffix_lens, prompt_len: int, tile: int, n_random: int, seed: int = 0, group: int = 0,
                rows_per_item: int = 256, item_bounds: Optional[int] = None) -> np.ndarray:
    """Packed token rows for sampled parity: per rollout the first and last row, the rows on
    both sides of the prompt/response boundary and of every multiple of `tile`, plus random rows.

    With `group` (= Hq / Hkv) also the positions around work-item boundaries: a work item covers
    `rows_per_item` stacked rows m = position * group + head-in-group, so item k starts inside position
    floor(k * rows_per_item / group); that position (whose heads may be split over two items) and its two
    neighbours are added, for every boundary of a rollout or, with `item_bounds` = n, for its first, its last
    and n seeded others."""
    rng = np.random.default_rng(seed + 12345)
    off = np.concatenate([[0], np.cumsum(np.asarray(suffix_lens, dtype=np.int64))])
    rows = []
    for g, S in enumerate(np.asarray(suffix_lens, dtype=np.int64)):
        S = int(S)
        local = {0, S - 1}
        if 0 < prompt_len < S:
            local.update({prompt_len - 1, prompt_len})
        for b in range(tile, S, tile):
            local.update({b - 1, b})
        local.update(int(x) for x in rng.integers(0, S, size=n_random))
        if group > 0:
            ks = np.arange(1, (S * group + rows_per_item - 1) // rows_per_item)
            if item_bounds is not None and len(ks) > item_bounds + 2:
                ks = np.concatenate([ks[:1], ks[-1:], rng.choice(ks[1:-1], size=item_bounds, replace=False)])
            for k in ks:
                p = int(k) * rows_per_item // group
                local.update(i for i in (p - 1, p, p + 1) if 0 <= i < S)
        rows.extend(int(off[g]) + i for i in sorted(local))
    return np.asarray(rows, dtype=np.int64)
