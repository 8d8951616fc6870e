"""CPU check of the tolerance model that the GPU gradient tests use for the error the bf16-rounded forward output
leaves in the backward (tests/gpu_util.delta_error_sigma).  The model is a statistical statement, so it is pinned
to a simulation rather than to itself: the gradients are computed from the definition in fp64 twice, once with
delta_i = <dO_i, O_i> from the exact O and once from O rounded to bf16 (everything else exact); the difference,
element by element, must be distributed like the predicted standard deviations."""
import numpy as np
import pytest

from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import delta_error_sigma


def grads_with_delta_from(x, d_out, round_out):
    """dQ, dK_prefix, dK_suffix from the definition (softmax Jacobian written out); delta taken from the exact
    output or from its bf16 rounding."""
    w = x.workload
    T, Hq, Hkv, D, P = x.total_suffix, w.num_q_heads, w.num_kv_heads, w.head_dim, w.prefix_len
    group = Hq // Hkv
    dq = np.zeros((T, Hq, D))
    dkp = np.zeros((P, Hkv, D))
    dks = np.zeros((T, Hkv, D))
    off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])
    f64 = lambda a: np.asarray(a, dtype=np.float64)
    for g in range(len(x.suffix_lens)):
        a, b = int(off[g]), int(off[g + 1])
        S = b - a
        for h in range(Hq):
            c = h // group
            keys = np.concatenate([f64(x.k_prefix[:, c]), f64(x.k_suffix[a:b, c])])
            vals = np.concatenate([f64(x.v_prefix[:, c]), f64(x.v_suffix[a:b, c])])
            q, do = f64(x.q[a:b, h]), f64(d_out[a:b, h])
            s = w.scale * (q @ keys.T)
            s[:, P:][np.triu(np.ones((S, S), dtype=bool), 1)] = -np.inf
            p = np.exp(s - s.max(axis=1, keepdims=True))
            p /= p.sum(axis=1, keepdims=True)
            o = p @ vals
            if round_out:
                o = f64(wl.round_to_bf16(o.astype(np.float32))[1])
            delta = np.sum(do * o, axis=1, keepdims=True)
            ds = p * (do @ vals.T - delta)
            dq[a:b, h] = w.scale * ds @ keys
            dk = w.scale * ds.T @ q
            dkp[:, c] += dk[:P]
            dks[a:b, c] += dk[P:]
    return {"dq": dq, "dk_prefix": dkp, "dk_suffix": dks}


@pytest.mark.parametrize("std,P,lens", [(1.0, 40, (30, 17)), (1.0, 1, (60, 45)), (2.5, 200, (120, 50)), (3.2, 0, (90, 3))])
def test_delta_error_model_matches_a_simulation(std, P, lens):
    x = wl.make_custom("bf16", 6, 2, 64, P, lens, seed=11, std=std)
    do, _ = wl.make_d_out(x)
    exact = grads_with_delta_from(x, do, round_out=False)
    rounded = grads_with_delta_from(x, do, round_out=True)
    sigma = delta_error_sigma(x, do)
    for name in ("dq", "dk_prefix", "dk_suffix"):
        err, sg = rounded[name] - exact[name], sigma[name]
        if err.size == 0:
            continue
        big = sg > 1e-3 * sg.max()                     # elements where the prediction is not vanishingly small
        z = err[big] / sg[big]
        print(f"{name}: {big.sum()} elements, rms of error / sigma = {np.sqrt(np.mean(z * z)):.2f}, max {np.abs(z).max():.2f}")
        # bf16 rounding errors are uniform inside a binade, i.e. within u/2 ... u of the value (u = 2^-8): the
        # model's u / sqrt 3 is their largest standard deviation and 0.74 of it the log-uniform average
        assert 0.6 <= np.sqrt(np.mean(z * z)) <= 0.9, name
        assert np.abs(z).max() <= 6.0, name
        assert np.abs(err[~big]).max(initial=0.0) <= 6.0 * 1e-3 * sg.max(), name


def test_delta_error_model_is_zero_for_fp32_and_small_for_many_keys():
    x32 = wl.make_custom("f32", 4, 2, 64, 10, (5, 3), seed=1)
    do32, _ = wl.make_d_out(x32)
    assert all(float(np.abs(v).max(initial=0.0)) == 0.0 for v in delta_error_sigma(x32, do32).values())
    x = wl.make_custom("bf16", 4, 2, 64, 2000, (40,), seed=2)
    do, _ = wl.make_d_out(x)
    sig = delta_error_sigma(x, do)
    exact = grads_with_delta_from(x, do, round_out=False)
    # with 2,000 visible keys the term is below the final rounding of the gradient itself (up to 2^-8 of its size)
    assert sig["dq"].max() < 0.5 * 2.0 ** -8 * np.sqrt(np.mean(exact["dq"] ** 2))
