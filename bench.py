#!/usr/bin/env python3
"""Benchmark of the prefix-shared GRPO prefill attention hot path on one MI355X.

One "step" = one pass of the whole hot path (prefix pass + suffix pass + merge + LSE export)
over one synthetic batch that is already resident in HBM.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3] [--no-cpu-baseline]
  python bench.py --direction backward ...   times prefix_attn_backward instead (see backward_main)

metric  : effective attention TFLOP/s = 4 D Hq sum_g[S_g P + S_g (S_g + 1) / 2] / time
roofline: the prefix pass (the dominant kernel) against the published dense bf16 MFMA peak
cpu_baseline: the fp64 C oracle on this host's cores, on a bounded sample of the same
          workload's query rows (also used as a parity spot check of the GPU result)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16 (published: 2.5 PFLOP/s)
HBM_PEAK_GBS = 8000.0


def measured_traffic(workload: str, kernel: str):
    """HBM bytes per launch of `kernel`, as measured with rocprofv3 hardware counters and recorded
    in the committed summary profiles/<kernel>_<workload>_hbm_traffic.txt (None if not recorded)."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":", 1)[1].split()[0]))
    except OSError:
        pass
    return None


def smi_sample():
    """Clocks and power as rocm-smi reports them right now (None if the tool is absent or fails).
    Not sampled under a profiler: its preloaded library initialises the GPU in every child process, and
    rocm-smi (a script started through `env`) would then replace a GPU-initialised process with another.
    The script is started as a direct child of this interpreter for the same reason."""
    import shutil
    import subprocess
    if any(k.startswith(("ROCPROF", "ROCP_", "ROCTRACER")) for k in os.environ):
        return None
    tool = shutil.which("rocm-smi")
    if tool is None:
        return None
    try:
        r = subprocess.run([sys.executable, os.path.realpath(tool), "--showclocks", "--showpower", "--showmaxpower",
                            "--json"], capture_output=True, text=True, timeout=20)
        card = next(iter(json.loads(r.stdout).values()))
        return {k.strip(" :"): v.strip("()") for k, v in card.items()}
    except Exception:
        return None


def gpu_state(torch, step, as_found):
    """The machine's state, not a tuning knob: clocks as found before the first launch, and sampled again
    while about half a second of the same steps is queued on the GPU (outside the timed region)."""
    if as_found is None:   # no rocm-smi here, or a profiler is attached: launch nothing extra
        return None
    t0 = time.perf_counter()
    step()
    torch.cuda.synchronize()
    n = max(1, min(2000, int(0.5 / max(time.perf_counter() - t0, 1e-4))))
    for _ in range(n):
        step()
    loaded = smi_sample()
    torch.cuda.synchronize()
    return {"as_found_idle": as_found, "under_load": loaded}


def calibrate_copy(torch):
    """Plain copy kernels of known size (256 MiB read, 256 MiB written each) for scaling traffic counters."""
    src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    for _ in range(3):
        torch.mul(src, 1.0, out=dst)
    torch.cuda.synchronize()


RECORD = ""


def emit(result):
    line = json.dumps(result)
    print(line, flush=True)
    if RECORD:
        with open(RECORD, "a") as f:
            f.write(line + "\n")


# What the `traffic` figure of a roofline block is: the committed counter summary of the same command, not a
# quantity of this run.  FETCH_SIZE / WRITE_SIZE count bytes that cross from the L2 caches to the fabric (L2
# misses and write-backs); the 256 MB memory-side cache may serve part of them, and no counter exposed by
# rocprofv3 here separates its hits, so the figure is an upper bound of the HBM bytes.
TRAFFIC_NOTE = "recorded rocprofv3 profile (profiles/), L2-miss + write-back bytes per launch: upper bound of HBM bytes"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C3")
    ap.add_argument("--direction", choices=("forward", "backward"), default="forward",
                    help="forward (default): the prefill attention hot path; backward: its gradient pass")
    ap.add_argument("--prefix-shards", type=int, default=0,
                    help="n > 0: time what ONE device of an n-way prefix-key-sharded group computes (its shard's "
                         "partial pass + the n-way merge); the exchange of partials between devices is not part of it")
    ap.add_argument("--logprob", default="", metavar="L3",
                    help="time the response-token log-probability path on this log-prob workload instead")
    ap.add_argument("--fold-prompt", action="store_true",
                    help="two-level sharing: the rollouts share their question, so the prompt is computed once and "
                         "joins the shared prefix (two calls per step); also times the one-call form on the same values")
    ap.add_argument("--prefix-frames", type=int, default=-1, metavar="F",
                    help="forward/backward: run the workload with a video prefix of F frames instead of its own "
                         "(same rollouts; for measuring how time depends on the prefix length)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    ap.add_argument("--power-probe", action="store_true",
                    help="after the timed region run the same launches on constant inputs (the same instruction stream "
                         "without operand toggling) and report time and shader clock of both")
    ap.add_argument("--record", default="", metavar="FILE", help="also append the JSON line to FILE")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed region also launch plain 256 MiB copy kernels (known HBM bytes, for "
                         "scaling hardware traffic counters under rocprofv3)")
    args = ap.parse_args()
    global RECORD
    RECORD = args.record
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2507_07966_amd as pa
    from paper_2507_07966_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    pa.load_library()   # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    args.smi_as_found = smi_sample()

    if args.logprob:
        return logprob_main(args, pa, wl, torch)

    if args.fold_prompt:
        return folded_main(args, pa, wl, torch)

    w = wl.WORKLOADS[args.workload]
    if args.prefix_frames >= 0:
        import dataclasses
        w = dataclasses.replace(w, frames=args.prefix_frames, name=f"{w.name}@{args.prefix_frames}frames",
                                note=f"{w.note}; prefix changed to {args.prefix_frames} frames")
    x = wl.make_inputs(w)
    T, P = x.total_suffix, w.prefix_len
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32

    def up(name):
        if w.dtype == "bf16":
            return torch.from_numpy(x.bits[name].view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(getattr(x, name)).cuda()

    dev = {n: up(n) for n in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")}
    t0 = time.perf_counter()
    plan = pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, P, x.suffix_lens, w.scale, dtype=w.dtype, device=0)
    plan_first_ms = (time.perf_counter() - t0) * 1e3    # includes loading the library's code object onto the device
    t0 = time.perf_counter()                            # what a training step with new rollout lengths pays
    pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, P, x.suffix_lens, w.scale, dtype=w.dtype, device=0).destroy()
    plan_ms = (time.perf_counter() - t0) * 1e3
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
    out = torch.empty((T, w.num_q_heads, w.head_dim), dtype=tdt, device="cuda")
    lse = torch.empty((w.num_q_heads, T), dtype=torch.float32, device="cuda")
    fwd_args = (plan, dev["q"], dev["k_prefix"] if P else None, dev["v_prefix"] if P else None, dev["k_suffix"],
                dev["v_suffix"], out, ws)

    def step():
        pa.prefix_attn_forward(*fwd_args)
        pa.prefix_attn_lse(plan, ws, lse)

    if args.prefix_shards > 0:
        return sharded_main(args, pa, wl, torch, w, x, dev, out, lse)
    if args.direction == "backward":
        step()
        return backward_main(args, pa, wl, torch, w, x, dev, plan, out, lse)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    per_step = np.array([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)])
    ms_per_step = float(ev[0].elapsed_time(ev[args.steps]) / args.steps)

    # per-kernel durations over the same number of steps (HIP events on the launch stream)
    kms = np.array([pa.prefix_attn_forward_timed(*fwd_args) for _ in range(args.steps)])
    k_prepass_ms, k_prefix_ms, k_suffix_ms, k_merge_ms = (float(v) for v in kms.mean(axis=0))

    if args.calibrate_copy:
        calibrate_copy(torch)
    state = gpu_state(torch, step, args.smi_as_found)

    flop = wl.effective_flop(w.num_q_heads, w.head_dim, P, x.suffix_lens)
    tflops = flop / (ms_per_step * 1e-3) * 1e-12
    prefix_flop = 4 * w.head_dim * w.num_q_heads * T * P
    suffix_flop = flop - prefix_flop
    if P and k_prefix_ms > 0.02:
        dom_name, dom_flop, dom_ms = "prefix_pass", prefix_flop, k_prefix_ms
    elif P:   # short prefix: the plan runs one sweep over [prefix | own keys] (timed in the suffix-pass slot)
        dom_name, dom_flop, dom_ms = "attention_sweep", flop, k_suffix_ms
    else:
        dom_name, dom_flop, dom_ms = "suffix_pass", suffix_flop, k_suffix_ms
    achieved = dom_flop / (dom_ms * 1e-3) * 1e-12
    e = 2 if w.dtype == "bf16" else 4
    merge_bytes = T * w.num_q_heads * (w.head_dim * ((8 if P else 4) + e) + (12 if P else 8))
    result = {
        "metric": "effective attention TFLOP/s",
        "value": round(tflops, 2),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.note}", "num_q_heads": w.num_q_heads, "num_kv_heads": w.num_kv_heads,
                   "head_dim": w.head_dim, "prefix_len": P, "prompt_len": w.prompt_len,
                   "num_rollouts": w.num_rollouts, "total_suffix_tokens": T,
                   "suffix_lens_min_max": [int(x.suffix_lens.min()), int(x.suffix_lens.max())]},
        "pct_of_bf16_mfma_peak": round(100 * tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "tokens_per_s_suffix": round(T / (ms_per_step * 1e-3), 1),
        "tokens_per_s_equiv_full_prefill": round(float(np.sum(P + x.suffix_lens.astype(np.int64))) / (ms_per_step * 1e-3), 1),
        "effective_flop": flop,
        "ms_median": round(float(np.median(per_step)), 4),
        "wall_ms_per_step": round(wall_ms / args.steps, 4),
        "plan_ms": round(plan_ms, 3),
        "plan_first_call_ms": round(plan_first_ms, 3),
        "kernel_ms": {"v_layout_prepass": round(k_prepass_ms, 4), "prefix_pass": round(k_prefix_ms, 4), "suffix_pass": round(k_suffix_ms, 4), "merge": round(k_merge_ms, 4)},
        # bf16 calls combine the two partials in the suffix pass's epilogue: no merge launch (its slot reads ~0)
        "merge_hbm_gbs": round(merge_bytes / (k_merge_ms * 1e-3) * 1e-9, 1) if k_merge_ms > 0.01 else None,
        "rocm_smi": state,
        "roofline": {"kernel": dom_name, "bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic(w.name, dom_name), "traffic_source": TRAFFIC_NOTE},
    }

    if not args.no_cpu_baseline:
        from oracle import cref
        rows_all = wl.sample_rows(x.suffix_lens, w.prompt_len, 256, 96, seed=1)
        rng = np.random.default_rng(2)
        rng.shuffle(rows_all)

        def run_oracle(rows):
            t = time.perf_counter()
            o, l, thr = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                     x.suffix_lens, w.scale, rows=rows)
            return o, l, thr, time.perf_counter() - t

        off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])

        def pairs_of(rows):
            g = np.searchsorted(off, rows, side="right") - 1
            return int(np.sum(P + (rows - off[g]) + 1))

        run_oracle(rows_all[:1])                       # warm the thread pool and the page cache
        probe = rows_all[:16]
        _, _, thr, t_probe = run_oracle(probe)
        n = int(max(16, min(len(rows_all), args.cpu_seconds / max(t_probe / len(probe), 1e-6))))
        rows = np.sort(rows_all[:n])
        o_ref, l_ref, thr, t_cpu = run_oracle(rows)
        cpu_flop = 4 * w.head_dim * w.num_q_heads * pairs_of(rows)
        o_gpu = out[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        l_gpu = lse[:, torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {
            "value": round(cpu_flop / t_cpu * 1e-12, 6), "unit": "TFLOP/s", "cores": int(thr), "kind": "oracle",
            "sample": f"{len(rows)} seeded query rows x {w.num_q_heads} heads of {w.name} against their full key sets "
                      f"(fp64, {t_cpu:.1f} s)",
            "seconds": round(t_cpu, 2),
            "extrapolated_full_workload_seconds": round(t_cpu * flop / cpu_flop, 1),
        }
        result["parity_on_sample"] = {"out_max_abs": float(np.abs(o_gpu - o_ref).max()),
                                      "out_mean_abs": float(np.abs(o_gpu - o_ref).mean()),
                                      "lse_max_abs": float(np.abs(l_gpu - l_ref).max())}
    if args.power_probe:
        result["power_probe"] = power_probe(args, pa, torch, plan, dev, out, ws, lse, ms_per_step, state)
    emit(result)


def power_probe(args, pa, torch, plan, dev, out, ws, lse, ms_random, state_random):
    """The same plan and launches on constant inputs: every operand of every MFMA is 1.0, so the instruction
    stream is identical but nothing toggles in the data path.  Time and sampled shader clock of both runs show
    how much of the step time is set by the power limit rather than by the schedule."""
    ones = {n: torch.ones_like(t) for n, t in dev.items()}
    P = plan.prefix_len
    cargs = (plan, ones["q"], ones["k_prefix"] if P else None, ones["v_prefix"] if P else None, ones["k_suffix"],
             ones["v_suffix"], out, ws)

    def cstep():
        pa.prefix_attn_forward(*cargs)
        pa.prefix_attn_lse(plan, ws, lse)

    for _ in range(args.warmup):
        cstep()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        cstep()
    e1.record()
    torch.cuda.synchronize()
    ms_const = float(e0.elapsed_time(e1) / args.steps)
    kms = np.array([pa.prefix_attn_forward_timed(*cargs) for _ in range(args.steps)]).mean(axis=0)
    state_const = gpu_state(torch, cstep, args.smi_as_found)

    def sclk(state):
        try:
            return state["under_load"]["sclk clock speed"]
        except (TypeError, KeyError):
            return None
    return {"random_inputs": {"ms_per_step": round(ms_random, 4), "sclk_under_load": sclk(state_random)},
            "constant_inputs": {"ms_per_step": round(ms_const, 4), "sclk_under_load": sclk(state_const),
                                "kernel_ms": [round(float(v), 4) for v in kms]},
            "time_ratio_random_over_constant": round(ms_random / ms_const, 4)}


def folded_main(args, pa, wl, torch):
    """The shared question folded into the prefix (prompt call + folded call per step) next to the one-call
    form on the same shared-prompt values; forward, or with --direction backward the gradient pass (whose dO
    values are arbitrary here: timing only, parity is the tests' job)."""
    backward = args.direction == "backward"
    w = wl.WORKLOADS[args.workload]
    x = wl.share_prompt(wl.make_inputs(w))
    prompt_call, folded_call, _ = wl.fold_prompt(x)

    def prepare(c):
        cw = c.workload
        dev = [torch.from_numpy(c.bits[n].view(np.int16)).cuda().view(torch.bfloat16)
               for n in ("q", "k_prefix", "v_prefix", "k_suffix", "v_suffix")]
        plan = pa.prefix_attn_plan(cw.num_q_heads, cw.num_kv_heads, cw.head_dim, cw.prefix_len, c.suffix_lens, cw.scale,
                                   dtype=cw.dtype, device=0)
        ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
        out = torch.empty((c.total_suffix, cw.num_q_heads, cw.head_dim), dtype=torch.bfloat16, device="cuda")
        lse = torch.empty((cw.num_q_heads, c.total_suffix), dtype=torch.float32, device="cuda")
        pa.prefix_attn_forward(plan, *dev, out, ws)
        pa.prefix_attn_lse(plan, ws, lse)
        bwd = None
        if backward:
            d_out = torch.randn(out.shape, dtype=torch.float32, device="cuda").to(torch.bfloat16)
            grads = [torch.empty_like(t) for t in dev]
            bws = torch.empty(plan.backward_workspace_bytes, dtype=torch.uint8, device="cuda")
            bwd = (d_out, grads, bws)
        return plan, dev, ws, out, lse, bwd

    def run(prepared):
        plan, dev, ws, out, lse, bwd = prepared
        if backward:
            d_out, grads, bws = bwd
            pa.prefix_attn_backward(plan, *dev, out, d_out, lse, *grads, bws)
        else:
            pa.prefix_attn_forward(plan, *dev, out, ws)
            pa.prefix_attn_lse(plan, ws, lse)

    def timed(calls):
        for _ in range(args.warmup):
            for c in calls:
                run(c)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            for c in calls:
                run(c)
        e1.record()
        torch.cuda.synchronize()
        return float(e0.elapsed_time(e1) / args.steps)

    two_level = [prepare(prompt_call), prepare(folded_call)]
    one_call = [prepare(x)]
    ms_fold = timed(two_level)
    ms_one = timed(one_call)
    count = wl.backward_flop if backward else wl.effective_flop
    flop_fold = sum(count(w.num_q_heads, w.head_dim, c.workload.prefix_len, c.suffix_lens)
                    for c in (prompt_call, folded_call))
    flop_one = count(w.num_q_heads, w.head_dim, w.prefix_len, x.suffix_lens)
    tflops = flop_fold / (ms_fold * 1e-3) * 1e-12
    emit({
        "metric": "effective attention backward TFLOP/s" if backward else "effective attention TFLOP/s",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_fold, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name} with one question shared by all rollouts, prompt folded into the prefix: "
                               f"call 1 = {w.prompt_len} prompt tokens over {w.prefix_len} video tokens, call 2 = prefix "
                               f"{w.prefix_len + w.prompt_len}, {w.num_rollouts} rollouts of response tokens only"},
        "pct_of_bf16_mfma_peak": round(100 * tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "effective_flop": flop_fold,
        "one_call_form": {"ms_per_step": round(ms_one, 4), "effective_flop": flop_one,
                          "tflops": round(flop_one / (ms_one * 1e-3) * 1e-12, 2)},
        "time_saved_pct": round(100 * (1 - ms_fold / ms_one), 2),
        "flop_saved_pct": round(100 * (1 - flop_fold / flop_one), 2),
    })


def logprob_main(args, pa, wl, torch):
    """One "step" = token_logprob_forward (LM-head GEMM tile kernel + finalize) for all response tokens of one
    question's rollouts under ONE model, inputs resident in HBM.  metric: 2 N d V / time."""
    w = wl.LOGPROB_WORKLOADS[args.logprob]
    x = wl.make_logprob_inputs(w)
    h = torch.from_numpy(x.bits["hidden"].view(np.int16)).cuda().view(torch.bfloat16)
    W = torch.from_numpy(x.bits["lm_head"].view(np.int16)).cuda().view(torch.bfloat16)
    y = torch.from_numpy(x.targets).cuda()
    N, d, V = w.num_tokens, w.hidden_dim, w.vocab
    ws = torch.empty(pa.token_logprob_workspace(N, d, V), dtype=torch.uint8, device="cuda")
    lp = torch.empty(N, dtype=torch.float32, device="cuda")
    lse = torch.empty(N, dtype=torch.float32, device="cuda")
    for _ in range(args.warmup):
        pa.token_logprob_forward(h, W, y, 1.0, lp, lse, ws)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        pa.token_logprob_forward(h, W, y, 1.0, lp, lse, ws)
    e1.record()
    torch.cuda.synchronize()
    ms = float(e0.elapsed_time(e1) / args.steps)
    flop = wl.logprob_flop(w)
    tflops = flop / (ms * 1e-3) * 1e-12
    result = {
        "metric": "LM-head log-probability TFLOP/s", "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.note}", "num_tokens": N, "hidden_dim": d, "vocab": V},
        "tokens_per_s": round(N / (ms * 1e-3), 1), "flop": flop,
        # the tile kernel is all but the microseconds of the finalize kernel
        "roofline": {"kernel": "logprob_tile", "bound": "mfma", "achieved": round(tflops, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(tflops / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic(w.name, "logprob_tile"), "traffic_source": TRAFFIC_NOTE},
    }
    if args.calibrate_copy:
        calibrate_copy(torch)
    if args.power_probe:   # the same launch on constant inputs (see power_probe)
        state_r = gpu_state(torch, lambda: pa.token_logprob_forward(h, W, y, 1.0, lp, lse, ws), args.smi_as_found)
        h1, W1 = torch.ones_like(h), torch.full_like(W, 2.0 ** -6)
        lp1, lse1 = torch.empty_like(lp), torch.empty_like(lse)
        cstep = lambda: pa.token_logprob_forward(h1, W1, y, 1.0, lp1, lse1, ws)
        for _ in range(args.warmup):
            cstep()
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(args.steps):
            cstep()
        c1.record()
        torch.cuda.synchronize()
        state_c = gpu_state(torch, cstep, args.smi_as_found)
        sclk = lambda st: st["under_load"].get("sclk clock speed") if st and st.get("under_load") else None
        result["power_probe"] = {"random_inputs": {"ms_per_step": round(ms, 4), "sclk_under_load": sclk(state_r)},
                                 "constant_inputs": {"ms_per_step": round(float(c0.elapsed_time(c1) / args.steps), 4),
                                                     "sclk_under_load": sclk(state_c)}}
    if not args.no_cpu_baseline:
        from oracle import ref_logprob
        idx = np.sort(np.random.default_rng(4).choice(N, size=min(N, 64), replace=False))
        t0 = time.perf_counter()
        rp, rl = ref_logprob.token_logprobs(x.hidden[idx], x.lm_head, x.targets[idx], 1.0)
        t_cpu = time.perf_counter() - t0
        try:
            cores = len(os.sched_getaffinity(0))
        except AttributeError:
            cores = os.cpu_count()
        got = lp[torch.from_numpy(idx).cuda()].cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {"value": round(2 * len(idx) * d * V / t_cpu * 1e-12, 6), "unit": "TFLOP/s",
                                  "cores": int(cores), "kind": "oracle",
                                  "sample": f"{len(idx)} seeded tokens against the whole vocabulary (fp64 numpy, {t_cpu:.1f} s)"}
        result["parity_on_sample"] = {"logprob_max_abs": float(np.abs(got - rp).max())}
    emit(result)


def sharded_main(args, pa, wl, torch, w, x, dev, out, lse):
    """One device's share when the P prefix keys are split into n shards (paper Sec. 5.2, sequence parallelism):
    a partial pass over P/n prefix keys (+ the rollouts' own keys on this device) for ALL suffix rows, then the
    n-way merge of the partials it would have received.  The other n-1 partials are produced here by the same
    device beforehand (untimed) so the merge reads real data."""
    n = args.prefix_shards
    T, P = x.total_suffix, w.prefix_len
    assert P % n == 0 and P > 0, "prefix_len must be divisible by the number of shards"
    Ps = P // n
    plan = pa.prefix_attn_plan(w.num_q_heads, w.num_kv_heads, w.head_dim, Ps, x.suffix_lens, w.scale, dtype=w.dtype, device=0)
    ws = torch.empty(plan.workspace_bytes, dtype=torch.uint8, device="cuda")
    po = [torch.empty((T, w.num_q_heads, w.head_dim), dtype=torch.float32, device="cuda") for _ in range(n)]
    pl = [torch.empty((T, w.num_q_heads), dtype=torch.float32, device="cuda") for _ in range(n)]

    def partial(i):
        a, b = i * Ps, (i + 1) * Ps
        pa.prefix_attn_forward_partial(plan, dev["q"], dev["k_prefix"][a:b], dev["v_prefix"][a:b],
                                       dev["k_suffix"] if i == 0 else None, dev["v_suffix"] if i == 0 else None,
                                       i == 0, po[i], pl[i], ws)

    for i in range(1, n):
        partial(i)

    def step():
        partial(0)
        pa.prefix_attn_merge_partials(plan, po, pl, out, lse)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    t_part = t_merge = 0.0
    for _ in range(args.steps):
        ev[0].record()
        partial(0)
        ev[1].record()
        pa.prefix_attn_merge_partials(plan, po, pl, out, lse)
        ev[2].record()
        torch.cuda.synchronize()
        t_part += ev[0].elapsed_time(ev[1])
        t_merge += ev[1].elapsed_time(ev[2])
    t_part /= args.steps
    t_merge /= args.steps
    ms = t_part + t_merge
    flop_dev = 4 * w.head_dim * w.num_q_heads * (T * Ps + wl.visible_pairs(0, x.suffix_lens))
    e = 2 if w.dtype == "bf16" else 4
    merge_bytes = T * w.num_q_heads * (n * (w.head_dim + 1) * 4 + w.head_dim * e + 4)
    result = {
        "metric": "effective attention TFLOP/s of one device in a prefix-sharded group (exchange excluded)",
        "value": round(flop_dev / (ms * 1e-3) * 1e-12, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "strong",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name} with the prefix keys in {n} shards: {w.note}", "prefix_shards": n,
                   "prefix_keys_per_shard": Ps, "total_suffix_tokens": T},
        "kernel_ms": {"shard_partial_pass_incl_suffix": round(t_part, 4), "merge_of_partials": round(t_merge, 4)},
        "roofline": {"kernel": "merge_partials", "bound": "hbm", "achieved": round(merge_bytes / (t_merge * 1e-3) * 1e-9, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(merge_bytes / (t_merge * 1e-3) * 1e-9 / HBM_PEAK_GBS, 4),
                     "traffic": None},
    }
    if args.calibrate_copy:
        calibrate_copy(torch)
    if not args.no_cpu_baseline:
        from oracle import cref
        rows = np.sort(wl.sample_rows(x.suffix_lens, w.prompt_len, 256, 2, seed=1))[:64]
        t0 = time.perf_counter()
        ro, rl, thr = cref.prefix_shared_attention(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix, x.suffix_lens,
                                                   w.scale, rows=rows)
        t_cpu = time.perf_counter() - t0
        off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])
        gi = np.searchsorted(off, rows, side="right") - 1
        cpu_flop = 4 * w.head_dim * w.num_q_heads * int(np.sum(P + (rows - off[gi]) + 1))
        o_gpu = out[torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        l_gpu = lse[:, torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
        result["cpu_baseline"] = {"value": round(cpu_flop / t_cpu * 1e-12, 6), "unit": "TFLOP/s", "cores": int(thr),
                                  "kind": "oracle", "sample": f"{len(rows)} seeded query rows x {w.num_q_heads} heads "
                                  f"against the whole (unsharded) key set (fp64, {t_cpu:.1f} s)"}
        result["parity_on_sample"] = {"out_max_abs": float(np.abs(o_gpu - ro).max()),
                                      "lse_max_abs": float(np.abs(l_gpu - rl).max())}
    emit(result)


def backward_main(args, pa, wl, torch, w, x, dev, plan, out, lse):
    """One "step" = one prefix_attn_backward call (pre-pass, dQ pass, dK/dV passes) on the outputs of a
    forward call, everything resident in HBM.  metric: 10 D Hq pairs / time (five products, each once)."""
    T, P = x.total_suffix, w.prefix_len
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    do_vals, do_bits = wl.make_d_out(x)
    if w.dtype == "bf16":
        do = torch.from_numpy(do_bits.view(np.int16)).cuda().view(torch.bfloat16)
    else:
        do = torch.from_numpy(do_vals).cuda()
    g = {"dq": torch.empty((T, w.num_q_heads, w.head_dim), dtype=tdt, device="cuda"),
         "dk_prefix": torch.empty((P, w.num_kv_heads, w.head_dim), dtype=tdt, device="cuda"),
         "dv_prefix": torch.empty((P, w.num_kv_heads, w.head_dim), dtype=tdt, device="cuda"),
         "dk_suffix": torch.empty((T, w.num_kv_heads, w.head_dim), dtype=tdt, device="cuda"),
         "dv_suffix": torch.empty((T, w.num_kv_heads, w.head_dim), dtype=tdt, device="cuda")}
    bws = torch.empty(max(plan.backward_workspace_bytes, 16), dtype=torch.uint8, device="cuda")
    has_p = P > 0
    bargs = (plan, dev["q"], dev["k_prefix"] if has_p else None, dev["v_prefix"] if has_p else None, dev["k_suffix"],
             dev["v_suffix"], out, do, lse, g["dq"], g["dk_prefix"] if has_p else None,
             g["dv_prefix"] if has_p else None, g["dk_suffix"], g["dv_suffix"], bws)
    for _ in range(args.warmup):
        pa.prefix_attn_backward(*bargs)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        pa.prefix_attn_backward(*bargs)
    e1.record()
    torch.cuda.synchronize()
    ms_per_step = float(e0.elapsed_time(e1) / args.steps)
    kms = np.array([pa.prefix_attn_backward_timed(*bargs) for _ in range(args.steps)]).mean(axis=0)
    if args.calibrate_copy:
        calibrate_copy(torch)
    power = None
    if args.power_probe:   # the same launches with every tensor set to 1.0 (see power_probe)
        state_r = gpu_state(torch, lambda: pa.prefix_attn_backward(*bargs), args.smi_as_found)
        cargs = tuple(torch.ones_like(t) if i in (1, 2, 3, 4, 5, 6, 7) and t is not None else t for i, t in enumerate(bargs))
        cargs = cargs[:8] + (torch.zeros_like(lse),) + cargs[9:]      # LSE of all-equal scores is not needed exactly
        for _ in range(args.warmup):
            pa.prefix_attn_backward(*cargs)
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(args.steps):
            pa.prefix_attn_backward(*cargs)
        c1.record()
        torch.cuda.synchronize()
        ckms = np.array([pa.prefix_attn_backward_timed(*cargs) for _ in range(args.steps)]).mean(axis=0)
        state_c = gpu_state(torch, lambda: pa.prefix_attn_backward(*cargs), args.smi_as_found)
        sclk = lambda st: st["under_load"].get("sclk clock speed") if st and st.get("under_load") else None
        power = {"random_inputs": {"ms_per_step": round(ms_per_step, 4), "sclk_under_load": sclk(state_r),
                                   "kernel_ms": [round(float(v), 4) for v in kms]},
                 "constant_inputs": {"ms_per_step": round(float(c0.elapsed_time(c1) / args.steps), 4),
                                     "sclk_under_load": sclk(state_c), "kernel_ms": [round(float(v), 4) for v in ckms]}}
    pairs = wl.visible_pairs(P, x.suffix_lens)
    flop = wl.backward_flop(w.num_q_heads, w.head_dim, P, x.suffix_lens)
    tflops = flop / (ms_per_step * 1e-3) * 1e-12
    # dominant kernel: the dK/dV pass over the prefix keys executes four products (S, dW, dV, dK) per pair
    if has_p:
        dom_name, dom_flop, dom_ms = "bwd_dkv_prefix", 8 * w.head_dim * w.num_q_heads * T * P, float(kms[2])
    else:
        dom_name, dom_flop, dom_ms = "bwd_dkv_suffix", 8 * w.head_dim * w.num_q_heads * pairs, float(kms[3])
    achieved = dom_flop / (dom_ms * 1e-3) * 1e-12
    result = {
        "metric": "effective attention backward TFLOP/s", "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name} backward: {w.note}", "num_q_heads": w.num_q_heads,
                   "num_kv_heads": w.num_kv_heads, "head_dim": w.head_dim, "prefix_len": P,
                   "num_rollouts": w.num_rollouts, "total_suffix_tokens": T},
        "pct_of_bf16_mfma_peak": round(100 * tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "effective_flop": flop,
        "kernel_ms": {"prepass": round(float(kms[0]), 4), "dq": round(float(kms[1]), 4),
                      "dkv_prefix": round(float(kms[2]), 4), "dkv_suffix": round(float(kms[3]), 4)},
        "executed_mfma_tflops": {"dq": round(6 * w.head_dim * w.num_q_heads * pairs / (kms[1] * 1e-3) * 1e-12, 1)},
        "roofline": {"kernel": dom_name, "bound": "mfma", "achieved": round(achieved, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic(w.name, dom_name), "traffic_source": TRAFFIC_NOTE},
    }
    if not args.no_cpu_baseline:
        from oracle import cref
        rows_all = wl.sample_rows(x.suffix_lens, w.prompt_len, 256, 96, seed=1)
        rng = np.random.default_rng(2)
        rng.shuffle(rows_all)

        def run_oracle(rows):
            t = time.perf_counter()
            dq_ref, thr = cref.prefix_shared_attention_backward(x.q, x.k_prefix, x.v_prefix, x.k_suffix, x.v_suffix,
                                                                x.suffix_lens, w.scale, do_vals, rows=rows)
            return dq_ref, thr, time.perf_counter() - t

        off = np.concatenate([[0], np.cumsum(x.suffix_lens.astype(np.int64))])
        run_oracle(rows_all[:1])
        probe = rows_all[:16]
        _, thr, t_probe = run_oracle(probe)
        n = int(max(16, min(len(rows_all), args.cpu_seconds / max(t_probe / len(probe), 1e-6))))
        rows = np.sort(rows_all[:n])
        dq_ref, thr, t_cpu = run_oracle(rows)
        gi = np.searchsorted(off, rows, side="right") - 1
        cpu_pairs = int(np.sum(P + (rows - off[gi]) + 1))
        cpu_flop = 6 * w.head_dim * w.num_q_heads * cpu_pairs     # the oracle's dQ rows: S, dW and dQ products
        dq_gpu = g["dq"][torch.from_numpy(rows).cuda()].float().cpu().numpy().astype(np.float64)
        rms = float(np.sqrt(np.mean(dq_ref * dq_ref)))
        result["cpu_baseline"] = {
            "value": round(cpu_flop / t_cpu * 1e-12, 6), "unit": "TFLOP/s", "cores": int(thr), "kind": "oracle",
            "sample": f"dQ of {len(rows)} seeded query rows x {w.num_q_heads} heads of {w.name} against their full key "
                      f"sets (fp64, {t_cpu:.1f} s)", "seconds": round(t_cpu, 2)}
        result["parity_on_sample"] = {"dq_max_abs_over_rms": float(np.abs(dq_gpu - dq_ref).max() / rms),
                                      "dq_mean_abs_over_rms": float(np.abs(dq_gpu - dq_ref).mean() / rms)}
    if power:
        result["power_probe"] = power
    emit(result)


if __name__ == "__main__":
    main()
