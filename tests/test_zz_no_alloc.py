"""prefix_attn_forward_static: the forward on the library's own static workspace (for callers that cannot
allocate).  Through the C ABI, against prefix_attn_forward + prefix_attn_lse on a caller-owned workspace (same
kernels, same schedule: bit for bit) and against the fp64 oracle; two calls in a row, the second smaller, so
whatever the first left in the shared array must not matter.  The file name makes pytest collect it
last: it runs after every other test has used the GPU, and alone in a fresh process when named on the command line."""
import numpy as np
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import check, run_hip, to_device


def run_static(x):
    import torch
    import paper_2507_07966_amd as pa
    w = x.workload
    dev = {n: to_device(x, n) for n in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    plan = pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, w.prefix_len, x.suffix_lens, w.scale,
                               dtype=w.dtype, device=0)
    assert plan.workspace_bytes <= pa.STATIC_SCRATCH_BYTES
    T = x.total_suffix
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    out = torch.full((T, w.num_q_heads, w.head_dim), float("nan"), device="cuda", dtype=tdt)
    lse = torch.full((w.num_q_heads, T), float("nan"), device="cuda", dtype=torch.float32)
    kp = dev["k_prefix"] if w.prefix_len > 0 else None
    vp = dev["v_prefix"] if w.prefix_len > 0 else None
    before = torch.cuda.memory_allocated()
    pa.prefix_attn_forward_static(plan, dev["q"], kp, vp, dev["k_suffix"], dev["v_suffix"], out, lse)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    plan.destroy()
    return out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)


@pytest.mark.gpu
def test_static_workspace_forward_two_calls_second_smaller():
    cases = [wl.make_custom("bf16", 2, 2, 64, 65600, (9000, 7600), seed=40),         # prefix pass + merging suffix pass
             wl.make_custom("bf16", 28, 4, 128, 700, (300, 129, 77), seed=41),       # smaller: one sweep
             wl.make_custom("bf16", 28, 4, 128, 5000, (40, 3), seed=42),             # prefix key ranges + n-way merge
             wl.make_custom("f32", 4, 2, 64, 100, (33, 70), seed=43)]                # fp32: stand-alone merge kernel
    import paper_2507_07966_amd as pa
    probe = pa.prefix_attn_plan(2, 2, 64, 65600, [9000, 7600], 64 ** -0.5, dtype="bf16", device=-1)
    assert len(probe.items(3)) == 0 and len(set(probe.items(0)[:, 5].tolist())) == 1   # no sweep, one key range
    probe.destroy()
    for x in cases:
        w = x.workload
        print(f"static workspace case {w.dtype} P={w.prefix_len} lens={x.suffix_lens.tolist()}", flush=True)
        out_s, lse_s = run_static(x)
        out_w, lse_w = run_hip(x)
        assert np.array_equal(out_s, out_w) and np.array_equal(lse_s, lse_w)
        ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, w.scale)
        check(out_s, lse_s, ro, rl, f"static workspace {w.dtype} P={w.prefix_len}")


@pytest.mark.gpu
def test_static_workspace_rejects_a_plan_that_does_not_fit():
    import torch
    import paper_2507_07966_amd as pa
    plan = pa.prefix_attn_plan(28, 4, 128, 4096, [1152] * 8, 128 ** -0.5, dtype="bf16", device=0)
    assert plan.workspace_bytes > pa.STATIC_SCRATCH_BYTES
    t = torch.zeros(64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(pa.PrefixAttnError) as e:
        pa.prefix_attn_forward_static(plan, t, t, t, t, t, t, None)
    assert e.value.status == 5      # PA_ERR_WORKSPACE, before anything is launched
    plan.destroy()


@pytest.mark.gpu
@pytest.mark.parametrize("Hq,Hkv,D,P,lens", [(28, 4, 128, 700, (300, 129, 77)),     # one sweep
                                              (28, 4, 128, 5000, (40, 3))])           # prefix key ranges + n-way merge
def test_static_workspace_forward_replays_in_a_captured_graph(Hq, Hkv, D, P, lens):
    """One of the callers the allocation-free entry point is for: a captured HIP graph.  The call is captured
    once and replayed three times, each time on new inputs copied into the same buffers, with the program's own
    eager work and synchronisations between the replays; every replay must equal, bit for bit, the eager call on
    the same inputs."""
    import torch
    import paper_2507_07966_amd as pa
    names = ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")
    x = wl.make_custom("bf16", Hq, Hkv, D, P, lens, seed=60)
    dev = {n: to_device(x, n) for n in names}
    plan = pa.prefix_attn_plan(Hq, Hkv, D, P, list(lens), x.workload.scale, dtype="bf16", device=0)
    assert plan.workspace_bytes <= pa.STATIC_SCRATCH_BYTES
    T = x.total_suffix
    out = torch.zeros((T, Hq, D), device="cuda", dtype=torch.bfloat16)
    lse = torch.zeros((Hq, T), device="cuda", dtype=torch.float32)

    def call():
        pa.prefix_attn_forward_static(plan, dev["q"], dev["k_prefix"], dev["v_prefix"], dev["k_suffix"],
                                      dev["v_suffix"], out, lse)

    call()                       # eager once: nothing is resolved or loaded for the first time under capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call()
    for seed in (61, 62, 63):
        xn = wl.make_custom("bf16", Hq, Hkv, D, P, lens, seed=seed)
        for n in names:
            dev[n].copy_(to_device(xn, n))
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        out_g, lse_g = out.clone(), lse.clone()
        out.fill_(float("nan"))
        lse.fill_(float("nan"))
        call()
        torch.cuda.synchronize()
        assert torch.isfinite(out_g.float()).all() and torch.isfinite(lse_g).all()
        assert torch.equal(out_g, out) and torch.equal(lse_g, lse), f"replay with seed {seed} differs from the eager call"
    plan.destroy()


def test_static_workspace_argument_checks_need_no_gpu():
    """The size limit is checked first, then the plan's device: both before anything touches a GPU."""
    import paper_2507_07966_amd as pa
    lib = pa.load_library()
    big = pa.prefix_attn_plan(28, 4, 128, 4096, [1152] * 8, 128 ** -0.5, dtype="bf16", device=-1)
    small = pa.prefix_attn_plan(28, 4, 128, 700, [40, 3], 128 ** -0.5, dtype="bf16", device=-1)
    assert big.workspace_bytes > pa.STATIC_SCRATCH_BYTES >= small.workspace_bytes
    p = 4096      # any aligned non-null value: no argument is dereferenced before the checks fail
    assert lib.prefix_attn_forward_static(big.handle, p, p, p, p, p, p, None, None) == 5       # PA_ERR_WORKSPACE
    assert lib.prefix_attn_forward_static(small.handle, p, p, p, p, p, p, None, None) == 3     # PA_ERR_UNSUPPORTED: host-only plan
    assert lib.prefix_attn_forward_static(None, p, p, p, p, p, p, None, None) == 1             # PA_ERR_NULL
