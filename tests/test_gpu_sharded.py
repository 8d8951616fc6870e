"""GPU parity of the composition over prefix-key shards: every shard's fp32 partial
(prefix_attn_forward_partial) combined by prefix_attn_merge_partials must reproduce the oracle's
attention over the whole prefix, to the same tolerances as the unsharded forward."""
import numpy as np
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import check, run_hip, to_device

pytestmark = pytest.mark.gpu


def run_sharded(x, bounds, suffix_shard=0):
    """bounds: prefix split points [0, b1, ..., P]; shard `suffix_shard` also covers the rollouts' own keys."""
    import torch
    import paper_2507_07966_amd as pa
    w = x.workload
    dev = {n: to_device(x, n) for n in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    T = x.total_suffix
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    parts_o, parts_l, plans = [], [], []
    for i in range(len(bounds) - 1):
        a, b = bounds[i], bounds[i + 1]
        plan = pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, b - a, x.suffix_lens, w.scale,
                                   dtype=w.dtype, device=0)
        ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
        o = torch.full((T, w.num_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device="cuda")
        l = torch.full((T, w.num_q_heads), float("nan"), dtype=torch.float32, device="cuda")
        with_suffix = i == suffix_shard
        pa.prefix_attn_forward_partial(plan, dev["q"], dev["k_prefix"][a:b] if b > a else None,
                                       dev["v_prefix"][a:b] if b > a else None,
                                       dev["k_suffix"] if with_suffix else None, dev["v_suffix"] if with_suffix else None,
                                       with_suffix, o, l, ws)
        parts_o.append(o)
        parts_l.append(l)
        plans.append(plan)
    out = torch.full((T, w.num_q_heads, w.head_dim), float("nan"), dtype=tdt, device="cuda")
    lse = torch.full((w.num_q_heads, T), float("nan"), dtype=torch.float32, device="cuda")
    pa.prefix_attn_merge_partials(plans[0], parts_o, parts_l, out, lse)
    torch.cuda.synchronize()
    for p in plans:
        p.destroy()
    return out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


CASES = [
    ("bf16", 28, 4, 128, 1000, (300, 77, 129), [0, 256, 700, 1000], 0),     # uneven shards, not tile multiples
    ("bf16", 28, 4, 128, 1000, (300, 77, 129), [0, 1000], 0),               # one shard: partial + merge == forward
    ("bf16", 14, 2, 64, 513, (100, 300), [0, 1, 2, 257, 513], 3),           # tiny shards; suffix on the last shard
    ("bf16", 8, 1, 128, 0, (65, 64), [0, 0], 0),                            # no prefix at all
    ("bf16", 8, 2, 128, 3000, (20, 9), [0, 1500, 3000], 1),                 # few rows: each shard's keys are split again inside the call
    # the shard with the own keys has more than 1,024 key tiles and enough rows to stay unsplit: prefix pass,
    # suffix pass and the two-way merge into an fp32 partial instead of one sweep
    ("bf16", 2, 2, 64, 66000, (9000, 7600), [0, 65800, 66000], 0),
    ("f32", 4, 2, 64, 100, (33, 70), [0, 30, 100], 1),
]


@pytest.mark.parametrize("dtype,Hq,Hkv,D,P,lens,bounds,suffix_shard", CASES)
def test_sharded_prefix_matches_oracle(dtype, Hq, Hkv, D, P, lens, bounds, suffix_shard):
    x = wl.make_custom(dtype, Hq, Hkv, D, P, lens, seed=21)
    print(f"sharded case {dtype} {Hq}/{Hkv}/{D} P={P} lens={lens} bounds={bounds}", flush=True)
    out, lse = run_sharded(x, bounds, suffix_shard)
    ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                             x.workload.scale)
    check(out, lse, ro, rl, f"sharded {bounds}")
    if dtype == "f32":
        assert np.abs(out - ro).max() < 1e-5 and np.abs(lse - rl).max() < 1e-5


def test_c3_eight_prefix_shards_sampled_rows():
    """The 32K-prefix workload split over 8 key shards of 4,096 (the shard a device of an 8-way
    sequence-parallel group would hold), merged on one device; sampled rows against the oracle."""
    w = wl.WORKLOADS["C3"]
    x = wl.make_inputs(w)
    bounds = list(range(0, w.prefix_len + 1, w.prefix_len // 8))
    out, lse = run_sharded(x, bounds)
    rows = wl.sample_rows(x.suffix_lens, w.prompt_len, 256, 4, seed=3)
    ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                             w.scale, rows=rows)
    check(out[rows], lse[:, rows], ro, rl, "C3 in 8 prefix shards")
    full_out, full_lse = run_hip(x)
    d = np.abs(out - full_out)
    print(f"sharded vs unsharded: out max {d.max():.3e} lse max {np.abs(lse - full_lse).max():.3e}", flush=True)
    assert d.max() <= 2e-2 and np.abs(lse - full_lse).max() <= 1e-4
