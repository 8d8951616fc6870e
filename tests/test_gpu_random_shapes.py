"""GPU parity on seeded random shapes (forward and backward, full tensors against the fp64 oracle): guards the
plan's choices (key splits for few rows, row splits for short prefixes) on shapes nobody hand-picked."""
import pytest

from oracle import cref
from paper_2507_07966_amd import workloads as wl
from tests.gpu_util import check, check_grads, delta_error_sigma, run_hip_backward
from tests.random_shapes import random_shapes

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("Hq,Hkv,D,P,lens", random_shapes())
def test_random_shape_forward_and_backward(Hq, Hkv, D, P, lens):
    x = wl.make_custom("bf16", Hq, Hkv, D, P, lens, seed=31)
    do, bits = wl.make_d_out(x)
    print(f"random shape Hq={Hq} Hkv={Hkv} D={D} P={P} lens={lens}", flush=True)
    got, (plan, args, _) = run_hip_backward(x, do, bits, keep=True)
    out, lse = args[6].float().cpu().numpy().astype("float64"), args[8].cpu().numpy().astype("float64")
    plan.destroy()
    a = (x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens, x.workload.scale)
    ro, rl, _ = cref.prefix_shared_attention(*a)
    check(out, lse, ro, rl, f"random {Hq}/{Hkv}/{D} P={P} {lens}")
    check_grads(got, cref.prefix_shared_attention_backward(*a, do)[:5], "bf16", f"random {Hq}/{Hkv}/{D} P={P} {lens}",
                sigmas=delta_error_sigma(x, do))
