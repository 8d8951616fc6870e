"""GPU parity: the HIP path (through the C ABI) against the fp64 oracle, element by element
on the same seeded inputs.  Tolerances: out max-abs <= 2e-2 and mean-abs <= 2e-3,
LSE max-abs <= 1e-3 (natural log)."""
import numpy as np
import pytest

from oracle import cref
from oracle import ref_attention as ref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import check, run_hip

pytestmark = pytest.mark.gpu


def oracle_full(x, scale=None):
    scale = x.workload.scale if scale is None else scale
    o, l, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, scale)
    return o, l


def test_c1_tiny_fp32_full_tensor():
    x = wl.make_inputs(wl.WORKLOADS["C1"])
    out, lse = run_hip(x)
    ro, rl = ref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, x.workload.scale)
    mx, _, ml = check(out, lse, ro, rl, "C1")
    assert mx < 1e-5 and ml < 1e-5      # fp32 arithmetic: far inside the bf16 tolerances


EDGE = [
    # dtype, Hq, Hkv, D, P, suffix_lens
    ("bf16", 28, 4, 128, 300, (70, 1, 129, 64)),     # ragged, P and S not multiples of any tile
    ("bf16", 28, 4, 128, 0, (200, 37)),              # no prefix: plain packed causal attention
    ("bf16", 4, 4, 128, 64, (1,)),                   # G = 1, S = 1, Hq = Hkv
    ("bf16", 8, 1, 128, 1, (65, 64, 63)),            # single prefix key, one kv head
    ("bf16", 14, 2, 64, 257, (100, 300)),            # head_dim 64
    ("bf16", 7, 1, 128, 1000, (37,) * 5),            # one GQA group, many short rollouts
    ("bf16", 2, 2, 128, 129, (513,)),                # rows cross several work items with group = 1
    ("bf16", 28, 4, 128, 5000, (40, 3)),             # few rows, long prefix: 9 key ranges, the last one ragged
    ("bf16", 8, 2, 64, 3000, (17,)),                 # the same with head_dim 64 (5 key ranges)
    ("bf16", 6, 3, 128, 300, (100, 57)),             # 3 kv heads do not divide the 8 XCDs: lists are not interleaved
    ("f32", 4, 2, 64, 100, (33, 70)),
    ("f32", 6, 2, 128, 0, (50, 1)),
    ("f32", 3, 3, 128, 65, (1, 2, 3)),
]


@pytest.mark.parametrize("dtype,Hq,Hkv,D,P,lens", EDGE)
def test_edge_shapes_full_tensor(dtype, Hq, Hkv, D, P, lens):
    x = wl.make_custom(dtype, Hq, Hkv, D, P, lens, seed=3)
    print(f"edge case {dtype} Hq={Hq} Hkv={Hkv} D={D} P={P} lens={lens}", flush=True)
    out, lse = run_hip(x)
    ro, rl = oracle_full(x)
    check(out, lse, ro, rl, f"edge {dtype} {Hq}/{Hkv}/{D} P={P} {lens}")


def test_long_prefix_takes_the_separate_passes_full_tensor():
    """A prefix of more than 1,024 tiles with enough rows to leave it unsplit: prefix pass, then the suffix pass
    that merges in its epilogue (shorter prefixes run as one sweep); head_dim 64, one head per kv head, ragged,
    full tensor."""
    import paper_2507_07966_amd as pa
    shape = (4, 4, 64, 65600, (3000, 2500, 2756))
    plan = pa.prefix_attn_plan(*shape[:4], list(shape[4]), 0.125, dtype="bf16", device=-1)
    assert len(plan.items(3)) == 0
    assert len(plan.items(0)) >= 129 and len(set(plan.items(0)[:, 4].tolist())) == 1        # unsplit prefix keys
    x = wl.make_custom("bf16", *shape, seed=13)
    out, lse = run_hip(x)
    ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                             x.workload.scale)
    check(out, lse, ro, rl, "long prefix, separate passes")


def test_graded_code_path_full_tensor():
    """Every element of the code path the 32K-prefix benchmark configuration takes: head_dim 128, 28 query heads
    over 4 kv heads (7 heads stacked per position), an unsplit prefix of more than 256 tiles with a ragged last
    tile, swept together with each block's own keys in one launch (the prefix part in the loop that carries no
    mask and no choice of key set); ragged rollouts, so blocks of rows end inside positions and rollouts."""
    import paper_2507_07966_amd as pa
    shape = (28, 4, 128, 16500, (700, 333, 517, 129, 650, 71))
    plan = pa.prefix_attn_plan(*shape[:4], list(shape[4]), 128 ** -0.5, dtype="bf16", device=-1)
    sw = plan.items(3)
    sw = sw[sw[:, 0] >= 0]
    assert len(sw) == sum((s * 7 + 255) // 256 for s in shape[4]) * 4 >= 256      # every block of rows once
    assert (sw[:, 4] == 0).all() and (sw[:, 5] == 16500).all()                    # each sweeps the whole prefix
    plan.destroy()
    x = wl.make_custom("bf16", *shape, seed=17)
    out, lse = run_hip(x)
    ro, rl = oracle_full(x)
    check(out, lse, ro, rl, "graded code path (D=128, group 7, one sweep over a 16.5K prefix and the own keys)")


def test_separate_passes_d128_group7_full_tensor():
    """The path of the hour-long and max-frame configurations, element by element: a prefix of more than 1,024
    tiles (ragged last tile) stays unsplit and runs as prefix pass + suffix pass with the merging epilogue,
    head_dim 128, 7 heads per kv head, ragged rollouts."""
    import paper_2507_07966_amd as pa
    shape = (28, 4, 128, 65700, (400, 333, 267, 200))
    plan = pa.prefix_attn_plan(*shape[:4], list(shape[4]), 128 ** -0.5, dtype="bf16", device=-1)
    pre = plan.items(0)
    pre = pre[pre[:, 0] >= 0]
    assert len(plan.items(3)) == 0                                                # no single sweep
    assert len(pre) == 140 and (pre[:, 4] == 0).all() and (pre[:, 3] == 65700).all()   # one key range: the whole prefix
    plan.destroy()
    x = wl.make_custom("bf16", *shape, seed=23)
    out, lse = run_hip(x)
    ro, rl = oracle_full(x)
    check(out, lse, ro, rl, "separate passes (D=128, group 7, unsplit 65.7K prefix + merging suffix pass)")


def test_large_scores_and_late_maximum():
    """Scores with a wide range, and the largest keys at the very end of the prefix, so the
    running reference maximum has to move late and by a lot."""
    x = wl.make_custom("bf16", 14, 2, 128, 700, (150, 90), seed=5, std=2.5)
    x.k_prefix[-3:] *= 3.0
    x.bits["k_prefix"], x.k_prefix = wl.round_to_bf16(x.k_prefix)
    out, lse = run_hip(x)
    ro, rl = oracle_full(x)
    check(out, lse, ro, rl, "late maximum")


def test_uniform_scores_give_mean_of_v_on_gpu():
    x = wl.make_custom("bf16", 4, 2, 128, 200, (30, 77), seed=6)
    x.q[...] = 0
    x.bits["q"][...] = 0
    out, lse = run_hip(x)
    off = ref.suffix_offsets(x.suffix_lens)
    for g in range(2):
        for i in (0, x.suffix_lens[g] - 1):
            t = off[g] + i
            for h in range(4):
                vis = np.concatenate([x.v_prefix[:, h // 2], x.v_suffix[off[g]:t + 1, h // 2]]).astype(np.float64)
                assert np.abs(out[t, h] - vis.mean(axis=0)).max() < 2e-3
                assert abs(lse[h, t] - np.log(200 + i + 1)) < 1e-4


def test_bitwise_reproducible():
    x = wl.make_custom("bf16", 28, 4, 128, 500, (300, 129), seed=7)
    a = run_hip(x)
    b = run_hip(x)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_c2_full_tensor():
    x = wl.make_inputs(wl.WORKLOADS["C2"])
    out, lse = run_hip(x)
    ro, rl = oracle_full(x)
    check(out, lse, ro, rl, "C2")


def test_non_default_stream_and_graph_replay():
    """forward + lse only enqueue work and allocate nothing, so they can run on any stream and be
    captured into a HIP graph; every replay must reproduce the eager result bit for bit."""
    import torch
    import paper_2507_07966_amd as pa
    from tests.gpu_util import to_device

    x = wl.make_custom("bf16", 28, 4, 128, 700, (300, 129), seed=9)
    w = x.workload
    eager_out, eager_lse = run_hip(x)
    dev = {n: to_device(x, n) for n in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    plan = pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, w.prefix_len, x.suffix_lens, w.scale,
                               dtype="bf16", device=0)
    T = x.total_suffix
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
    out = torch.zeros((T, 28, 128), dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros((28, T), dtype=torch.float32, device="cuda")

    def enqueue():
        pa.prefix_attn_forward(plan, dev["q"], dev["k_prefix"], dev["v_prefix"], dev["k_suffix"], dev["v_suffix"], out, ws)
        pa.prefix_attn_lse(plan, ws, lse)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue()
    side.synchronize()
    assert np.array_equal(out.float().cpu().numpy(), eager_out) and np.array_equal(lse.cpu().numpy(), eager_lse)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue()
    for rep in range(3):
        out.zero_()
        lse.zero_()
        ws.random_(0, 255)          # stale workspace contents must not matter
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.float().cpu().numpy(), eager_out), f"replay {rep}"
        assert np.array_equal(lse.cpu().numpy().astype(np.float64), eager_lse), f"replay {rep}"
    plan.destroy()
