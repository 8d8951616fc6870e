"""GPU parity of the response-token log-probabilities (and group advantages) against the fp64 oracle.
Tolerance: 1e-3 absolute on logprob and LSE (natural log), the bar used for the attention LSE; the
arithmetic (exact bf16 products, fp32 accumulation over the hidden dimension, fp32 log-sum-exp)
lands near 1e-5."""
import numpy as np
import pytest

from oracle import ref_logprob as ref
from paper_2507_07966_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-3


def run_hip(hidden_bits, head_bits, targets, scale=1.0, want_lse=True, junk_workspace=False):
    import torch
    import paper_2507_07966_amd as pa
    h = torch.from_numpy(hidden_bits.view(np.int16)).cuda().view(torch.bfloat16)
    w = torch.from_numpy(head_bits.view(np.int16)).cuda().view(torch.bfloat16)
    y = torch.from_numpy(np.ascontiguousarray(targets, dtype=np.int32)).cuda()
    N, d, V = h.shape[0], h.shape[1], w.shape[0]
    ws = torch.empty(pa.token_logprob_workspace(N, d, V), dtype=torch.uint8, device="cuda")
    if junk_workspace:      # finite, plausible-looking floats (0.5 ... 2) in every word
        ws.view(torch.int32).random_(0x3F000000, 0x40000000)
    lp = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    lse = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
    pa.token_logprob_forward(h, w, y, scale, lp, lse, ws)
    torch.cuda.synchronize()
    return lp.cpu().numpy().astype(np.float64), (lse.cpu().numpy().astype(np.float64) if want_lse else None)


def custom(N, d, V, seed, head_std=0.05):
    w = wl.LogprobWorkload("custom", N, d, V, head_std=head_std, seed=seed)
    return wl.make_logprob_inputs(w)


@pytest.mark.parametrize("N,d,V,scale", [
    (333, 512, 5000, 1.0),        # ragged in tokens and vocabulary
    (1, 64, 1, 1.0),              # one token, one-word vocabulary: logprob = 0
    (257, 128, 257, 0.7),         # one past a tile in both dimensions, temperature != 1
    (256, 64, 256, 1.0),          # exactly one tile
    (40, 192, 70000, 2.0),        # fewer than 8 token tiles: vocabulary tiles are split over the XCDs
    (2100, 64, 300, 1.0),         # more than 8 token tiles
])
def test_logprob_small_shapes_full(N, d, V, scale):
    x = custom(N, d, V, seed=N + V)
    # put some targets on tile and block borders
    edges = [v for v in (0, 31, 32, 63, 64, 255, 256, V - 1) if v < V]
    x.targets[:len(edges)] = np.array(edges[:N], dtype=np.int32)[:len(x.targets[:len(edges)])]
    print(f"logprob case N={N} d={d} V={V} scale={scale}", flush=True)
    lp, lse = run_hip(x.bits["hidden"], x.bits["lm_head"], x.targets, scale)
    rp, rl = ref.token_logprobs(x.hidden, x.lm_head, x.targets, scale)
    print(f"  logprob max-abs {np.abs(lp - rp).max():.3e}  lse max-abs {np.abs(lse - rl).max():.3e}", flush=True)
    assert np.isfinite(lp).all() and np.isfinite(lse).all()
    assert np.abs(lp - rp).max() <= TOL and np.abs(lse - rl).max() <= TOL


def test_logprob_peaked_and_wide_logits():
    """Logits with a wide range (std about 8): the running maximum matters."""
    x = custom(300, 256, 3000, seed=5, head_std=0.5)
    lp, lse = run_hip(x.bits["hidden"], x.bits["lm_head"], x.targets, 1.0)
    rp, rl = ref.token_logprobs(x.hidden, x.lm_head, x.targets, 1.0)
    assert np.abs(lp - rp).max() <= TOL and np.abs(lse - rl).max() <= TOL


def test_logprob_target_outside_the_vocabulary_gives_nan_not_a_stale_value():
    """Ids outside [0, V) (an ignore index on a padded slot, an id past the vocabulary) have no logit: their
    logprob must be NaN, whatever the workspace held before; their LSE and every other token are unaffected."""
    x = custom(300, 128, 1000, seed=8)
    y = x.targets.copy()
    bad = np.array([0, 17, 255, 256, 299])
    y[bad] = np.array([-100, -1, 1000, 1 << 30, -(1 << 31)], dtype=np.int64).astype(np.int32)
    lp, lse = run_hip(x.bits["hidden"], x.bits["lm_head"], y, 1.0, junk_workspace=True)
    rp, rl = ref.token_logprobs(x.hidden, x.lm_head, x.targets, 1.0)
    good = np.setdiff1d(np.arange(300), bad)
    assert np.isnan(lp[bad]).all()
    assert np.abs(lp[good] - rp[good]).max() <= TOL and np.abs(lse - rl).max() <= TOL


def test_logprob_7b_head_1000_tokens_full():
    x = wl.make_logprob_inputs(wl.LOGPROB_WORKLOADS["L2"])
    lp, lse = run_hip(x.bits["hidden"], x.bits["lm_head"], x.targets, 1.0)
    rp, rl = ref.token_logprobs(x.hidden, x.lm_head, x.targets, 1.0)
    print(f"L2: logprob max-abs {np.abs(lp - rp).max():.3e}  lse max-abs {np.abs(lse - rl).max():.3e}", flush=True)
    assert np.abs(lp - rp).max() <= TOL and np.abs(lse - rl).max() <= TOL


def test_logprob_full_size_sampled_tokens_and_bitwise_reproducible():
    """The benchmark shape (16,384 tokens x 152,064 words): 192 sampled tokens against the oracle; the
    result does not depend on which other tokens share the batch, and is bitwise reproducible."""
    x = wl.make_logprob_inputs(wl.LOGPROB_WORKLOADS["L3"])
    lp, lse = run_hip(x.bits["hidden"], x.bits["lm_head"], x.targets, 1.0)
    assert np.isfinite(lp).all()
    idx = np.unique(np.concatenate([[0, 255, 256, len(lp) - 1], np.random.default_rng(3).integers(0, len(lp), 188)]))
    rp, rl = ref.token_logprobs(x.hidden[idx], x.lm_head, x.targets[idx], 1.0)
    print(f"L3 sample of {len(idx)}: logprob max-abs {np.abs(lp[idx] - rp).max():.3e}", flush=True)
    assert np.abs(lp[idx] - rp).max() <= TOL and np.abs(lse[idx] - rl).max() <= TOL
    lp2, _ = run_hip(x.bits["hidden"], x.bits["lm_head"], x.targets, 1.0, want_lse=False)
    assert np.array_equal(lp, lp2)


def test_group_advantages():
    import torch
    import paper_2507_07966_amd as pa
    rng = np.random.default_rng(1)
    r = rng.random((37, 8)).astype(np.float32)
    r[3] = 0.5                      # a group without signal
    r[4] = [1, 0, 0, 1, 1, 0, 0, 1]
    dr = torch.from_numpy(r).cuda()
    out = torch.full_like(dr, float("nan"))
    pa.grpo_group_advantages(dr, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = np.stack([ref.group_advantages(g) for g in r])
    assert np.abs(got - want).max() < 1e-5
    assert (got[3] == 0).all()
