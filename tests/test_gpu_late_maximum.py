"""GPU parity on inputs whose softmax reference has to move late and by a lot, in every variant of the bf16
attention passes.

The forward takes a tile's probabilities against the maximum of a row's first tile and only checks, from the
tile's row sum, that they stay in a safe range; rows that leave it are redone by the second kernel of the pass
with a full online softmax.  N(0,1)-like scores never need that, so these cases construct it: wide scores
(std 2.5) and the largest keys at the very end of the prefix and of every rollout's own keys.  One case per
variant of the pass (one sweep, separate prefix and merging suffix pass, prefix keys split into ranges with the
n-way merge, shard partials with and without the own keys), at both head dimensions."""
import numpy as np
import pytest

from oracle import cref
from oracle import ref_attention as ref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import LSE_MAX_ABS, OUT_MEAN_ABS, run_hip

pytestmark = pytest.mark.gpu

SAFE_LOG2 = 16.0   # the kernel accepts a tile while its probabilities stay below 2^16 of the reference


def late_maximum_inputs(Hq, Hkv, D, P, lens, seed):
    x = wl.make_custom("bf16", Hq, Hkv, D, P, lens, seed=seed, std=2.5)
    off = ref.suffix_offsets(x.suffix_lens)
    if P >= 3:
        x.k_prefix[-3:] *= 3.0
        x.bits["k_prefix"], x.k_prefix = wl.round_to_bf16(x.k_prefix)
    for g in range(len(lens)):
        x.k_suffix[off[g + 1] - 2:off[g + 1]] *= 3.0
    x.bits["k_suffix"], x.k_suffix = wl.round_to_bf16(x.k_suffix)
    return x


def check_peaked(out, lse, ref_out, ref_lse, x, label):
    """Mean error and LSE to the bar of the other parity tests; the elementwise bound follows the magnitude.  These
    rows are close to one-hot, so an output element is close to one value |v| of up to 5, where bf16 is coarse:
    storing the result costs up to 2^-8 |ref| (half a bf16 spacing), rounding the probabilities to bf16 for the PV
    product up to 2^-8 sum_j p_j |v_j| <= 2^-8 max |v|; 1e-3 covers the fp32 arithmetic."""
    vmax = max(float(np.abs(x.v_prefix).max()) if x.v_prefix.size else 0.0, float(np.abs(x.v_suffix).max()))
    d = np.abs(out - ref_out)
    dl = np.abs(lse - ref_lse)
    excess = (d - (2.0 ** -8 * np.abs(ref_out) + 2.0 ** -8 * vmax + 1e-3)).max()
    msg = (f"{label}: out max-abs {d.max():.3e} mean-abs {d.mean():.3e}, largest excess over the elementwise bound "
           f"{excess:.3e}; lse max-abs {dl.max():.3e}")
    print(msg, flush=True)
    assert excess <= 0 and d.mean() <= OUT_MEAN_ABS and dl.max() <= LSE_MAX_ABS, msg


def rows_that_move(x, keys, rows):
    """How many of the (row, head) pairs of query rows `rows` see, among `keys` [n, Hkv, D] taken in order, a key
    after the first 64 that scores more than 2^16 times the maximum of the first 64 (in probability)."""
    w = x.workload
    group = w.num_q_heads // w.num_kv_heads
    n = 0
    for t in rows:
        for h in range(w.num_q_heads):
            s = keys[:, h // group].astype(np.float64) @ x.q[t, h].astype(np.float64) * w.scale * np.log2(np.e)
            n += int(len(s) > 64 and s[64:].max() - s[:64].max() > SAFE_LOG2)
    return n


CASES = [
    # (Hq, Hkv, D, P, lens, sweep expected, compare every n-th row (1: the full tensor))
    (8, 2, 64, 700, (150, 90), True, 1),          # one sweep, D = 64
    # more than 1,024 prefix tiles and more than 128 blocks of rows: unsplit prefix pass + merging suffix pass
    # (a row costs the oracle 65,700 keys: every 6th row, and the first and last 8 rows of every rollout)
    (28, 4, 128, 65700, (400, 333, 267, 200), False, 6),
    (16, 4, 64, 65700, (600, 500, 500, 500), False, 6),
    (8, 2, 128, 3000, (90, 70), False, 1),        # few rows: prefix keys in ranges, plain suffix partial, n-way merge
    (14, 2, 64, 66000, (150, 90), False, 1),      # the same with long ranges (4,416 keys each), D = 64
]


@pytest.mark.parametrize("Hq,Hkv,D,P,lens,sweep,every", CASES)
def test_late_maximum_in_every_forward_variant(Hq, Hkv, D, P, lens, sweep, every):
    import paper_2507_07966_amd as pa
    print(f"late maximum {Hq}/{Hkv}/{D} P={P} lens={lens}", flush=True)
    plan = pa.prefix_attn_plan(Hq, Hkv, D, P, list(lens), D ** -0.5, dtype="bf16", device=-1)
    assert (len(plan.items(3)) > 0) == sweep
    plan.destroy()
    x = late_maximum_inputs(Hq, Hkv, D, P, lens, seed=31)
    off = ref.suffix_offsets(x.suffix_lens)
    for g in range(len(lens)):                 # the inputs do what they are built for, on both key sets
        last = range(off[g + 1] - 4, off[g + 1])
        assert rows_that_move(x, x.k_prefix, last) > 0
        assert rows_that_move(x, x.k_suffix[off[g]:off[g + 1]], last) > 0
    out, lse = run_hip(x)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    rows = set(range(0, x.total_suffix, every))
    for g in range(len(lens)):
        rows |= set(range(off[g], off[g] + 8)) | set(range(off[g + 1] - 8, off[g + 1]))
    rows = np.array(sorted(rows))
    ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                             x.workload.scale, rows=rows)
    check_peaked(out[rows], lse[:, rows], ro, rl, x, f"late maximum D={D} P={P}")


@pytest.mark.parametrize("D", [128, 64])
def test_late_maximum_in_shard_partials(D):
    """Shard 0 holds prefix keys only (prefix pass leaving an fp32 partial), shard 1 its prefix keys and the
    rollouts' own keys (one sweep leaving an fp32 partial)."""
    from tests.test_gpu_sharded import run_sharded
    print(f"late maximum, shard partials D={D}", flush=True)
    x = late_maximum_inputs(14, 2, D, 1000, (150, 90), seed=32)
    x.k_prefix[397:400] *= 3.0                 # also at the end of shard 0
    x.bits["k_prefix"], x.k_prefix = wl.round_to_bf16(x.k_prefix)
    assert rows_that_move(x, x.k_prefix[:400], range(4)) > 0 and rows_that_move(x, x.k_prefix[400:], range(4)) > 0
    out, lse = run_sharded(x, [0, 400, 1000], suffix_shard=1)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    ro, rl, _ = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                             x.workload.scale)
    check_peaked(out, lse, ro, rl, x, f"late maximum, shard partials D={D}")
