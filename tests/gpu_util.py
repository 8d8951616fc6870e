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


GRAD_NAMES = ("dq", "dk_prefix", "dv_prefix", "dk_suffix", "dv_suffix")
# Gradient tolerances.  An element may be off by
#   |err| <= GRAD_REL * |ref| + GRAD_ABS_RMS * rms(ref),   and   mean|err| <= GRAD_MEAN_RMS * rms(ref).
# bf16 path: (1) every gradient is rounded to bf16 once at the end: relative 2^-9 of the element
# (GRAD_REL leaves a factor 2); (2) the weights W and dS are rounded to bf16 before the two
# accumulating products: independent relative 2^-9 errors, a few 1e-3 of the tensor's rms after
# summation; (3) delta = <dO, O> is taken from the bf16-rounded forward output, which perturbs
# every dS of a row by W * (2^-9-level error of a length-D dot product); it matters for rows that
# see only a few keys, where it reaches a few percent of the tensor's rms.  The mean bound is the
# sharp one (an ideal rounding of the exact gradient alone gives about 1.1e-3 rms).
GRAD_REL = {"bf16": 2.0 ** -8, "f32": 1e-5}
GRAD_ABS_RMS = {"bf16": 8e-2, "f32": 1e-4}
GRAD_MEAN_RMS = {"bf16": 3e-3, "f32": 1e-5}


def run_hip_backward(x, d_out, d_out_bits=None, scale=None, keep=False):
    """forward + backward through the C ABI.  Returns a dict name -> float64 array (and the forward out)."""
    import torch
    import paper_2507_07966_amd as pa
    w = x.workload
    scale = w.scale if scale is None else scale
    out64, lse64, plan, dev, ws, out, lse = run_hip(x, scale, return_plan=True)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    if w.dtype == "bf16":
        do = torch.from_numpy(d_out_bits.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        do = torch.from_numpy(d_out).cuda()
    T, P = x.total_suffix, w.prefix_len
    nan = float("nan")
    g = {"dq": torch.full((T, w.num_q_heads, w.head_dim), nan, dtype=tdt, device="cuda"),
         "dk_prefix": torch.full((P, w.num_kv_heads, w.head_dim), nan, dtype=tdt, device="cuda"),
         "dv_prefix": torch.full((P, w.num_kv_heads, w.head_dim), nan, dtype=tdt, device="cuda"),
         "dk_suffix": torch.full((T, w.num_kv_heads, w.head_dim), nan, dtype=tdt, device="cuda"),
         "dv_suffix": torch.full((T, w.num_kv_heads, w.head_dim), nan, dtype=tdt, device="cuda")}
    bws = torch.empty(max(plan.backward_workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    has_p = P > 0
    args = (plan, dev["q"], dev["k_prefix"] if has_p else None, dev["v_prefix"] if has_p else None, dev["k_suffix"],
            dev["v_suffix"], out, do, lse, g["dq"], g["dk_prefix"] if has_p else None, g["dv_prefix"] if has_p else None,
            g["dk_suffix"], g["dv_suffix"], bws)
    pa.prefix_attn_backward(*args)
    torch.cuda.synchronize()
    res = {n: t.float().cpu().numpy().astype(np.float64) for n, t in g.items()}
    if keep:
        return res, (plan, args, g)
    plan.destroy()
    return res


def check_grad_tensor(a, r, dtype, label=""):
    """One gradient tensor `a` against the oracle's `r` (same shape, last axis = head_dim).  Returns the worst
    element error in units of the tensor's rms."""
    assert a.shape == r.shape, f"{label}: shape {a.shape} vs {r.shape}"
    if r.size == 0:
        return 0.0
    assert np.isfinite(a).all(), f"{label}: non-finite gradient"
    rms = float(np.sqrt(np.mean(r * r)))
    d = np.abs(a - r)
    row = np.sqrt(np.mean(r * r, axis=-1, keepdims=True))        # rms of each (token, head) vector
    excess = np.maximum(d - GRAD_REL[dtype] * np.abs(r), 0.0)
    in_row_units = float((excess / np.maximum(row, 1e-3 * rms + 1e-300)).max())
    beyond = float(np.maximum(excess - 2.0 ** -5 * row, 0.0).max() / max(rms, 1e-300))
    msg = (f"{label}: max-abs {d.max():.3e} mean-abs {d.mean():.3e} (reference rms {rms:.3e}); worst element "
           f"{d.max() / max(rms, 1e-300):.3e} of the tensor's rms, {in_row_units:.3e} of its vector's rms, "
           f"beyond {beyond:.3e}")
    print(msg, flush=True)
    assert (d <= GRAD_REL[dtype] * np.abs(r) + GRAD_ABS_RMS[dtype] * rms + 1e-30).all(), msg
    assert d.mean() <= GRAD_MEAN_RMS[dtype] * rms + 1e-30, msg
    return d.max() / max(rms, 1e-30)


def check_grads(got, ref, dtype, label=""):
    """got: dict from run_hip_backward; ref: the oracle's five arrays in GRAD_NAMES order."""
    return max(check_grad_tensor(got[n], r, dtype, f"{label} {n}") for n, r in zip(GRAD_NAMES, ref))
