"""Helpers of the two-level sharing tests (shared prompt folded into the prefix): arranging the results of
the two calls in the unfolded reading.  No attention arithmetic: `backward(inputs, d_out)` is whichever
implementation the test examines and returns (dq, dk_prefix, dv_prefix, dk_suffix, dv_suffix)."""
import numpy as np

from paper_2507_07966_amd import workloads as wl


def unfold_rows(rows, folded, prompt):
    """Arrange per-row results of the two calls in the packed row order of the unfolded inputs."""
    return np.where((rows >= 0).reshape((-1,) + (1,) * (folded.ndim - 1)), folded[np.maximum(rows, 0)],
                    prompt[np.maximum(-rows - 1, 0)])


def args(x):
    return x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, x.workload.scale


def folded_backward(backward, x, d_out):
    """Gradients in the unfolded reading, computed through the two-level arrangement with `backward`."""
    p, f, rows = wl.fold_prompt(x)
    Lp, P = x.workload.prompt_len, x.workload.prefix_len
    resp = rows >= 0
    do_f = d_out[resp]
    do_p = np.zeros(p.q.shape, dtype=np.float64)
    np.add.at(do_p, -rows[~resp] - 1, d_out[~resp])         # the shared prompt rows collect every rollout's dO
    gf = backward(f, do_f)[:5]
    gp = backward(p, do_p)[:5]
    return {"dq_resp": gf[0], "dq_prompt": gp[0],
            "dk_video": gf[1][:P] + gp[1], "dv_video": gf[2][:P] + gp[2],
            "dk_prompt": gf[1][P:] + gp[3], "dv_prompt": gf[2][P:] + gp[4],
            "dk_resp": gf[3], "dv_resp": gf[4]}


def unfolded_backward(backward, x, d_out):
    _, _, rows = wl.fold_prompt(x)
    Lp = x.workload.prompt_len
    resp = rows >= 0
    dq, dkp, dvp, dks, dvs = backward(x, d_out)[:5]

    def prompt_sum(a):
        s = np.zeros((Lp,) + a.shape[1:], dtype=np.float64)
        np.add.at(s, -rows[~resp] - 1, a[~resp])
        return s
    return {"dq_resp": dq[resp], "dq_prompt": prompt_sum(dq), "dk_video": dkp, "dv_video": dvp,
            "dk_prompt": prompt_sum(dks), "dv_prompt": prompt_sum(dvs), "dk_resp": dks[resp], "dv_resp": dvs[resp]}


