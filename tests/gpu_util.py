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
# Gradient tolerances, from the rounding model of the bf16 path.  bf16 keeps 8 significant bits: rounding a value
# m * 2^e (1 <= m < 2) moves it by at most u |2^e| with u = 2^-8, uniformly, i.e. by a relative error uniform in
# [-u/m, u/m]: standard deviation at most BF16_SIGMA = u / sqrt 3 = 2.3e-3 (at m = 1), 0.74 of that over a
# mantissa that is spread log-uniformly (1.7e-3).  tests/test_tolerance_model.py checks these figures, and the
# delta term below, against a simulation.
# Every gradient vector (one token or key, one head, D channels) is a sum  y_d = sum_k a_k b_kd  whose factor a_k
# (a softmax weight W or a dS) was rounded to bf16 first.  Its error therefore has standard deviation
# 1.7e-3 sqrt(sum_k a_k^2 b_kd^2), and for factors b of mixed sign that root is the size of the vector's own
# elements: sigma = 1.7e-3 of the vector's root-mean-square, 6 sigma = 1.0e-2 at the largest of 1e8 elements
# (measured: 6e-3 ... 1.2e-2 on iid inputs, 1.7e-2 where all keys of a head share a mean vector, which cancels in
# the exact sum but not in the rounding errors).  The final rounding of the result adds at most u |y_d|.
# An element may therefore be off by
#   |err| <= GRAD_REL |ref| + GRAD_VEC rms(its vector) + GRAD_FLOOR rms(tensor),
# with GRAD_REL = u, GRAD_VEC = 2^-5 (three times the 6 sigma figure, 1.8 times the largest measured value), and
# the mean error by GRAD_MEAN_RMS rms(tensor) (the mean |error| of the model is 0.8 sigma = 1.3e-3, the final
# rounding adds as much again in quadrature; measured 1.4 ... 2.1e-3).
# The floor covers vectors that are small by cancellation, where the model's "own size" is not the error's
# scale: delta = <dO, O> is taken from the bf16-rounded forward output, an absolute error of about
# BF16_SIGMA sqrt(D) rms(dO) rms(O) on every dS of the row times its weight.  It is negligible next to the
# vector term once a row sees many keys (|O| ~ 1 / sqrt(keys)); for a key seen by a single row (rank-one dK) it
# reaches 2e-3 of the tensor's rms (floor 2^-7).  For rows that see one or two keys (or whose softmax is peaked),
# the exact dQ cancels to (almost) zero, |O| ~ rms(V), and the error of dQ = scale * sum_j dS_j k_j is the delta
# error times scale |k|: BF16_SIGMA scale sqrt(D) rms(dO) rms(V) |k_d| at one sigma, an ABSOLUTE size set by the
# inputs and not by the gradient tensor (a long rollout in the same call shrinks the tensor's rms, not this
# error).  delta_error_sigma() works this term out element by element from the definition (small shapes);
# few_keys_floor() is its closed form for rows with one or two keys: DELTA_SIGMAS of it at the largest |k_d| or
# |q_d| (the same term reaches dK through q), 6e-2 at N(0,1) inputs, measured 1.3e-2 ... 3.1e-2; it is added only
# when some row sees fewer than FEW_KEYS keys.
# fp32 path: fp32 rounding throughout.
BF16_SIGMA = 2.0 ** -8 / np.sqrt(3.0)
GRAD_REL = {"bf16": 2.0 ** -8, "f32": 1e-5}
GRAD_VEC = {"bf16": 2.0 ** -5, "f32": 1e-4}
GRAD_FLOOR = {"bf16": 2.0 ** -7, "f32": 1e-4}
FEW_KEYS = 8
DELTA_SIGMAS = 6.0
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


def few_keys_floor(x, d_out, scale=None):
    """Absolute tolerance term for calls in which some row sees fewer than FEW_KEYS keys (0.0 otherwise, and on
    the fp32 path): DELTA_SIGMAS standard deviations of the error that the bf16-rounded forward output leaves in
    delta, carried into dQ and dK (see the model above)."""
    w = x.workload
    if w.dtype != "bf16" or w.prefix_len + 1 >= FEW_KEYS:
        return 0.0
    scale = w.scale if scale is None else scale
    v = np.concatenate([x.v_prefix.ravel(), x.v_suffix.ravel()]).astype(np.float64)
    big = max(float(np.abs(x.q).max()), float(np.abs(x.k_suffix).max()),
              float(np.abs(x.k_prefix).max()) if x.k_prefix.size else 0.0)
    return float(DELTA_SIGMAS * BF16_SIGMA * scale * np.sqrt(w.head_dim) * np.sqrt(np.mean(np.square(d_out, dtype=np.float64)))
                 * np.sqrt(np.mean(v * v)) * big)


def delta_error_sigma(x, d_out, scale=None):
    """Per-element absolute tolerance for what the bf16-rounded forward output leaves in the gradients, worked
    out from the definition for small shapes (the weights P are formed explicitly in fp64).  The backward takes
    delta_i = <dO_i, O_i> from `out` as the forward wrote it, i.e. rounded to bf16: independent relative errors
    of standard deviation at most BF16_SIGMA on its elements, so delta_i is off by eps_i with standard deviation
        s_i <= BF16_SIGMA sqrt(sum_d dO_id^2 O_id^2).
    dS_ij = P_ij (dP_ij - delta_i) carries -P_ij eps_i into
        dQ_i = scale sum_j dS_ij k_j :  error  scale eps_i (sum_j P_ij k_j)            (one term)
        dK_j = scale sum_i dS_ij q_i :  error  scale sum_i eps_i P_ij q_i               (independent terms)
    Where the softmax of a row is spread over many keys both are far below the rounding of the gradient itself
    (|O_i| and |sum_j P_ij k_j| shrink like 1 / sqrt(keys)); where it is peaked, or the row sees one or two keys,
    the exact dQ_i cancels to almost zero while this error stays, so it has to be allowed for in absolute terms.
    dV has no such term.  Returns the standard deviations {"dq": [T,Hq,D], "dk_prefix": [P,Hkv,D],
    "dk_suffix": [T,Hkv,D]} (zeros on the fp32 path); check_grad_tensor() allows DELTA_SIGMAS of them per
    element, as few_keys_floor() does for its special case, and their mean in the mean error."""
    w = x.workload
    scale = w.scale if scale is None else scale
    T, Hq, Hkv, D, P = x.total_suffix, w.num_q_heads, w.num_kv_heads, w.head_dim, w.prefix_len
    tol = {"dq": np.zeros((T, Hq, D)), "dk_prefix": np.zeros((P, Hkv, D)), "dk_suffix": np.zeros((T, Hkv, D))}
    if w.dtype != "bf16":
        return tol
    group = Hq // Hkv
    var_kp = np.zeros((P, Hkv, D))
    var_ks = np.zeros((T, Hkv, D))
    off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    for g in range(len(x.suffix_lens)):
        a, b = int(off[g]), int(off[g + 1])
        S = b - a
        causal = np.tril(np.ones((S, S), dtype=bool))
        for h in range(Hq):
            c = h // group
            keys = np.concatenate([f64(x.k_prefix[:, c]), f64(x.k_suffix[a:b, c])])      # [P + S, D]
            vals = np.concatenate([f64(x.v_prefix[:, c]), f64(x.v_suffix[a:b, c])])
            q = f64(x.q[a:b, h])
            sc = scale * (q @ keys.T)
            sc[:, P:][~causal] = -np.inf
            sc -= sc.max(axis=1, keepdims=True)
            pr = np.exp(sc)
            pr /= pr.sum(axis=1, keepdims=True)
            o = pr @ vals
            do = f64(d_out[a:b, h])
            s_eps = BF16_SIGMA * np.sqrt(np.sum(do * do * o * o, axis=1))          # [S]
            tol["dq"][a:b, h] = scale * s_eps[:, None] * np.abs(pr @ keys)
            var = scale * scale * ((pr * s_eps[:, None]) ** 2).T @ (q * q)               # [P + S, D]
            var_kp[:, c] += var[:P]
            var_ks[a:b, c] += var[P:]
    tol["dk_prefix"] = np.sqrt(var_kp)
    tol["dk_suffix"] = np.sqrt(var_ks)
    return tol


def check_grad_tensor(a, r, dtype, label="", abs_floor=0.0, sigma=None):
    """One gradient tensor `a` against the oracle's `r` (same shape, last axis = head_dim).  abs_floor: what
    few_keys_floor() returned for the call; sigma: this tensor's array from delta_error_sigma(), if the test
    works that model out.  Returns the worst element error in units of its tolerance."""
    assert a.shape == r.shape, f"{label}: shape {a.shape} vs {r.shape}"
    if r.size == 0:
        return 0.0
    assert np.isfinite(a).all(), f"{label}: non-finite gradient"
    rms = float(np.sqrt(np.mean(r * r)))
    d = np.abs(a - r)
    vec = np.sqrt(np.mean(r * r, axis=-1, keepdims=True))        # rms of each (token or key, head) vector
    tol = GRAD_REL[dtype] * np.abs(r) + GRAD_VEC[dtype] * vec + GRAD_FLOOR[dtype] * rms + abs_floor + 1e-30
    mean_tol = GRAD_MEAN_RMS[dtype] * rms + 1e-30
    if sigma is not None:
        tol = tol + DELTA_SIGMAS * sigma
        mean_tol += float(np.mean(sigma))
    worst = float((d / tol).max())
    msg = (f"{label}: max-abs {d.max():.3e} mean-abs {d.mean():.3e} (reference rms {rms:.3e}); worst element at "
           f"{worst:.2f} of its tolerance, mean at {d.mean() / mean_tol:.2f}")
    print(msg, flush=True)
    assert worst <= 1.0, msg
    assert d.mean() <= mean_tol, msg
    return worst


def check_grads(got, ref, dtype, label="", abs_floor=0.0, sigmas=None):
    """got: dict from run_hip_backward; ref: the oracle's five arrays in GRAD_NAMES order; abs_floor: what
    few_keys_floor() returned for the call's inputs; sigmas: the dict from delta_error_sigma(), if used."""
    sigmas = sigmas or {}
    return max(check_grad_tensor(got[n], r, dtype, f"{label} {n}", abs_floor, sigmas.get(n))
               for n, r in zip(GRAD_NAMES, ref))
