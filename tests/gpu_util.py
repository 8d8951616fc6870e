"""Helpers for the GPU parity tests: upload seeded inputs, run the C-ABI path, compare."""
import numpy as np

OUT_MAX_ABS = 2e-2    # tolerances of the acceptance bar (max-abs / mean-abs on out, max-abs on LSE)
OUT_MEAN_ABS = 2e-3
LSE_MAX_ABS = 1e-3


def to_device(x, name):
    import torch
    w = x.workload
    if w.dtype == "bf16":
        return torch.from_numpy(x.bits[name].view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(getattr(x, name)).cuda()


def run_hip(x, scale=None, return_plan=False):
    """Run plan + forward + lse through the C ABI.  Returns out [T,Hq,D] float64, lse [Hq,T] float64."""
    import torch
    import paper_2507_07966_amd as pa
    w = x.workload
    scale = w.scale if scale is None else scale
    names = ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")
    dev = {n: to_device(x, n) for n in names}
    plan = pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, w.prefix_len, x.suffix_lens, scale,
                               dtype=w.dtype, device=0)
    T = x.total_suffix
    ws = torch.empty(max(plan.workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    out = torch.full((T, w.num_q_heads, w.head_dim), float("nan"), device="cuda",
                     dtype=torch.bfloat16 if w.dtype == "bf16" else torch.float32)
    lse = torch.full((w.num_q_heads, T), float("nan"), device="cuda", dtype=torch.float32)
    kp = dev["k_prefix"] if w.prefix_len > 0 else None
    vp = dev["v_prefix"] if w.prefix_len > 0 else None
    pa.prefix_attn_forward(plan, dev["q"], kp, vp, dev["k_suffix"], dev["v_suffix"], out, ws)
    pa.prefix_attn_lse(plan, ws, lse)
    torch.cuda.synchronize()
    res = out.float().cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    if return_plan:
        return res + (plan, dev, ws, out, lse)
    plan.destroy()
    return res


def check(out, lse, ref_out, ref_lse, label=""):
    assert np.isfinite(out).all(), f"{label}: non-finite output"
    assert np.isfinite(lse).all(), f"{label}: non-finite LSE"
    d = np.abs(out - ref_out)
    dl = np.abs(lse - ref_lse)
    msg = f"{label}: out max-abs {d.max():.3e} mean-abs {d.mean():.3e}; lse max-abs {dl.max():.3e}"
    print(msg, flush=True)
    assert d.max() <= OUT_MAX_ABS, msg
    assert d.mean() <= OUT_MEAN_ABS, msg
    assert dl.max() <= LSE_MAX_ABS, msg
    return d.max(), d.mean(), dl.max()
