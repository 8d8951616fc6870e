"""Turn rocprofv3 CSV output into the short text summaries kept under profiles/.

  python -m paper_2507_07966_amd.profile_summary stats   <..._kernel_stats.csv>
  python -m paper_2507_07966_amd.profile_summary counter <..._counter_collection.csv> [--copy-bytes N]

`counter` averages every collected counter per kernel.  For FETCH_SIZE / WRITE_SIZE it also
scales the reading by what the same counter shows for the plain copy kernels that
`bench.py --calibrate-copy` launches (each reads and writes --copy-bytes, default 256 MiB),
which turns counter units into bytes without trusting the documented unit.
"""
from __future__ import annotations

import collections
import csv
import re
import sys


def short_name(k: str) -> str:
    # mangled template arguments: <head_dim, causal, epilogue, sweep, careful> / <head_dim, causal, partial> / <head_dim, partial>
    if "pass_bf16_kernel" in k:
        m = re.search(r"pass_bf16_kernelILi\d+ELb(\d)ELi(\d)ELb(\d)ELb(\d)E", k)
        if m is None:
            return "attention pass (bf16 MFMA)"
        causal, epi, sweep, careful = (int(v) for v in m.groups())
        if careful:     # second launch of every pass: redoes the items the common kernel gave up on (none, normally)
            return "careful kernel of the " + ("prefix pass" if not causal else "sweep" if sweep else "suffix pass")
        if not causal:
            return "prefix_pass (bf16 MFMA)"
        if sweep:
            return "attention_sweep (bf16 MFMA)" + (", fp32 partial" if epi == 0 else "")
        return "suffix_pass (bf16 MFMA)" + ("" if epi == 0 else ", final" if epi == 1 else ", merging")
    if "bwd_dkv_reduce" in k:
        return "bwd_dkv: add partial gradients"
    if "bwd_dq_reduce" in k:
        return "bwd_dq: add key splits"
    if "bwd_dkv_kernel" in k:      # <head_dim, masked, partial gradients>
        if "ELb1ELb0E" in k:
            return "bwd_dkv_suffix (bf16 MFMA)"
        if "ELb1ELb1E" in k:
            return "bwd_dkv_suffix (bf16 MFMA), masked tiles, partials"
        # mask-free: the prefix keys, or (with partial gradients) their row splits and a long rollout's own keys
        return "bwd_dkv mask-free (bf16 MFMA), partials" if "ELb0ELb1E" in k else "bwd_dkv_prefix (bf16 MFMA)"
    if "bwd_dq_kernel" in k:
        return "bwd_dq (bf16 MFMA)" + (", key splits" if "ELb1E" in k else "")
    if "bwd_prep" in k:
        return "bwd_prepass"
    if "bwd_dq_f32" in k or "bwd_dkv_f32" in k or "bwd_delta_f32" in k:
        return "backward (fp32) " + ("dq" if "dq" in k else "dkv" if "dkv" in k else "delta")
    if "logprob_tile_kernel" in k:
        return "logprob_tile (bf16 MFMA)"
    if "logprob_finalize" in k:
        return "logprob_finalize"
    if "pass_f32_kernel" in k:
        return "attention pass (fp32)"
    if "merge_n_kernel" in k:
        return "merge_partials (n-way)"
    if "merge_kernel" in k:
        return "merge"
    if "vt_image_kernel" in k:      # <head_dim, key order of the 32x32x16 products>: the backward's images of K
        # (rocprofv3 prints short names demangled, long ones mangled)
        return "k_layout_prepass (backward)" if re.search(r"vt_image_kernel(ILi\d+ELb1E|<\d+, true>)", k) else "v_layout_prepass"
    if "lse_export" in k:
        return "lse_export"
    if "elementwise" in k and "Mul" in k or "mul" in k.lower() and "elementwise" in k:
        return "plain copy kernel (torch mul by 1)"
    return k[:60]


def stats(path: str) -> None:
    print(f"{'kernel':40s} {'calls':>6s} {'avg_us':>12s} {'min_us':>12s} {'max_us':>12s} {'pct':>7s}")
    for r in csv.DictReader(open(path)):
        print(f"{short_name(r['Name']):40s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:12.2f} "
              f"{float(r['MinNs']) / 1e3:12.2f} {float(r['MaxNs']) / 1e3:12.2f} {float(r['Percentage']):7.2f}")


def counter(path: str, copy_bytes: int) -> None:
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        agg[short_name(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    means = {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in agg.items()}
    for k, d in means.items():
        n = len(next(iter(agg[k].values())))
        print(f"{k:40s} dispatches={n:3d} " + " ".join(f"{c}={v:.6g}" for c, v in sorted(d.items())))
    copy = next((d for k, d in means.items() if k.startswith("plain copy kernel")), None)
    if copy:
        for c in ("FETCH_SIZE", "WRITE_SIZE"):
            if c in copy and copy[c] > 0:
                scale = copy_bytes / copy[c]
                print(f"\n{c}: the copy kernel moves {copy_bytes} bytes and reads {copy[c]:.6g} counter units "
                      f"=> {scale:.4f} bytes per unit")
                for k, d in means.items():
                    if c in d:
                        print(f"  {k:40s} {c} = {d[c] * scale / 1e6:12.2f} MB per dispatch")


if __name__ == "__main__":
    if len(sys.argv) < 3 or sys.argv[1] not in ("stats", "counter"):
        sys.exit(__doc__)
    if sys.argv[1] == "stats":
        stats(sys.argv[2])
    else:
        cb = int(sys.argv[sys.argv.index("--copy-bytes") + 1]) if "--copy-bytes" in sys.argv else 256 * 1024 * 1024
        counter(sys.argv[2], cb)
