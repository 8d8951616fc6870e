"""GPU parity of two-level sharing: with the same question for all G rollouts (Sec. 4.2) the prompt is
computed once (one call: prefix = video, suffix = prompt) and joins the shared prefix of a second call whose
rollouts hold their response tokens only.  The oracle evaluates the plain definition on the unfolded inputs
(every rollout attends to [video | its prompt copy | its response]); the HIP path runs the two calls."""
import numpy as np
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl
from tests.fold_util import args, folded_backward, unfold_rows, unfolded_backward
from tests.gpu_util import GRAD_FLOOR, GRAD_MEAN_RMS, GRAD_REL, GRAD_VEC, check, run_hip, run_hip_backward

pytestmark = pytest.mark.gpu

SHAPE = wl.Workload("F2", "bf16", 28, 4, 128, 20, 64, 100, 4, None, response_range=(200, 700), seed=4,
                    note="1,280 video tokens, a 100-token question shared by 4 ragged rollouts")


def test_folded_forward_matches_oracle_of_unfolded_definition():
    x = wl.share_prompt(wl.make_inputs(SHAPE))
    p, f, rows = wl.fold_prompt(x)
    ref_out, ref_lse, _ = cref.prefix_shared_attention(*args(x))
    po, pl = run_hip(p)
    fo, fl = run_hip(f)
    check(unfold_rows(rows, fo, po), unfold_rows(rows, fl.T, pl.T).T, ref_out, ref_lse, "two-level forward")


def test_folded_backward_matches_oracle_of_unfolded_definition():
    x = wl.share_prompt(wl.make_inputs(SHAPE))
    d_out, _ = wl.make_d_out(x, grid=1 / 8)       # multiples of 1/8: the sum over 4 rollouts is exact in bf16

    def hip_backward(inp, do):
        bits, back = wl.round_to_bf16(np.asarray(do, dtype=np.float32))
        assert np.array_equal(back, do), "dO must be exact in bf16"
        g = run_hip_backward(inp, back, bits)
        return tuple(g[n] for n in ("dq", "dk_prefix", "dv_prefix", "dk_suffix", "dv_suffix"))

    def oracle_backward(inp, do):
        return cref.prefix_shared_attention_backward(*args(inp), do)[:5]
    got = folded_backward(hip_backward, x, d_out)
    ref = unfolded_backward(oracle_backward, x, d_out)
    for n, r in ref.items():
        # gradients of the video and prompt tokens are sums of two bf16 results: twice the single-tensor tolerances
        k = 2.0 if n.endswith(("_video", "_prompt")) and n != "dq_prompt" else 1.0
        rms = float(np.sqrt(np.mean(r * r)))
        d = np.abs(got[n] - r)
        msg = f"two-level backward {n}: max-abs {d.max():.3e} mean-abs {d.mean():.3e} (reference rms {rms:.3e})"
        print(msg, flush=True)
        assert np.isfinite(got[n]).all(), msg
        vec = np.sqrt(np.mean(r * r, axis=-1, keepdims=True))
        assert (d <= k * (GRAD_REL["bf16"] * np.abs(r) + GRAD_VEC["bf16"] * vec + GRAD_FLOOR["bf16"] * rms)).all(), msg
        assert d.mean() <= k * GRAD_MEAN_RMS["bf16"] * rms, msg
