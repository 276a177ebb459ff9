#!/usr/bin/env python3
"""Every benchmark configuration in one table.

Runs ``bench.py`` once per workload (the small ones warm and cold) as child processes, collects their JSON
lines and prints a markdown report: step time, tokens/s, the dominant kernel's time and roofline fraction, the CPU
oracle's time on the same inputs, and the parity sample of the same run.

    python bench_all.py [--steps K] [--warmup W] [--out report.md] [--json lines.jsonl]

The small workloads (contexts of 128 to 2048 tokens) fit the 256 MB last-level cache; their fraction of the HBM peak is
quoted from the cold run (pools rotated through at least 512 MB), the warm run is what a serving loop over one
pool would see.  The long-context workloads are always cold.
"""
from __future__ import annotations

import argparse
import json
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))

# (workload, extra bench.py flags, also run cold, label)
RUNS = [
    ("decode_fp32_single", [], True, "1 fp32 decode 1 x 128, 8/8 heads, d 64"),
    ("decode_b8_ctx128", [], True, "2 bf16 decode 8 x 128, 32/8 heads"),
    ("decode_b8_ctx256", [], True, "2 bf16 decode 8 x 256"),
    ("decode_b8_ctx512", [], True, "2 bf16 decode 8 x 512"),
    ("decode_b8_ctx1024", [], True, "2 bf16 decode 8 x 1024"),
    ("decode_b8_ctx2048", [], True, "2 bf16 decode 8 x 2048"),
    ("prefill_b4_s2048_causal", [], True, "3 bf16 causal prefill 4 x 2048, 32/8 heads"),
    ("decode_mixed64_shared_prefix", ["--oracle-seqs", "64"], False, "4 bf16 decode, 64 seqs 64..32768, shared prefixes"),
    ("decode_b16_ctx131072_p16", ["--oracle-seqs", "16"], False, "5 bf16 decode 16 x 131072, 64/8 heads, P 16"),
    ("decode_b16_ctx131072_p64", ["--oracle-seqs", "16"], False, "5 same, P 64"),
    ("decode_b16_ctx131072_p16", ["--dtype", "fp16", "--oracle-seqs", "4"], False, "5 with fp16 pools"),
    ("decode_b16_ctx131072_p16", ["--head-dim", "64", "--oracle-seqs", "4"], False, "5 with head_dim 64"),
    ("decode_b16_ctx131072_p16", ["--head-dim", "256", "--oracle-seqs", "2"], False, "5 with head_dim 256"),
    ("prefill_b4_s2048_causal", ["--head-dim", "64"], False, "3 with head_dim 64"),
    ("prefill_b4_s2048_causal", ["--head-dim", "256"], False, "3 with head_dim 256"),
    ("paper_llama7b_decode_ctx128", [], True, "paper's setting: LLaMA-7B layer (32/32 heads, fp16, P 64), decode 1 x 128"),
    ("paper_llama7b_decode_ctx2048", [], True, "same, decode 1 x 2048"),
    ("paper_llama7b_prefill_s2048", [], True, "same, causal prefill of a 2048-token prompt"),
    ("contiguous_read_calibration", [], False, "yardstick: plain contiguous read of 8.59 GB"),
]


def run_one(workload, extra, cold, steps, warmup):
    cmd = [sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, "--steps", str(steps), "--warmup",
           str(warmup), "--no-prefill", *extra]
    if cold:
        cmd.append("--cold")
    r = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT)
    if r.returncode != 0:
        raise SystemExit(f"bench.py failed for {workload}:\n{r.stdout}\n{r.stderr}")
    line = [ln for ln in r.stdout.splitlines() if ln.startswith("{")][-1]
    print(f"done: {workload}{' (cold)' if cold else ''}", file=sys.stderr, flush=True)
    return json.loads(line)


def fmt_row(label, cache, j):
    roof = j.get("roofline", {})
    kern = roof.get("kernel", "")
    kern_us = j.get("kernels", {}).get(kern, {}).get("avg_us")
    cpu = j.get("cpu_baseline")
    par = j.get("parity_sample")
    frac = f"{100 * roof['frac']:.1f} % of {roof['peak']:g} {roof['unit']}" if roof else "-"
    if roof.get("bound") == "hbm" and roof.get("algorithmic_bytes", 0) < (2 << 20):
        frac += " (launch-bound: under 2 MB)"
    cells = [label, cache, f"{j['value']:.1f}", f"{j.get('tokens_per_s', 0):.3g}" if "tokens_per_s" in j else "-",
             f"{kern.replace('paged_', '').replace('_kernel', '')} {kern_us:.1f}" if kern_us else "-", frac,
             f"{cpu['value'] / 1e6:.3g} s on {cpu['cores']} cores ({cpu['sample'].split(' in ')[0]})" if cpu else "-",
             f"{par['max_abs']:.1e} / {par['max_rel_rms_floored']:.1e}" if par else "-"]
    return "| " + " | ".join(cells) + " |"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--out", default="")
    ap.add_argument("--json", default="")
    args = ap.parse_args()
    lines, rows = [], []
    for workload, extra, both, label in RUNS:
        big = workload.startswith(("decode_b16", "contiguous"))
        steps = min(args.steps, 20) if big else args.steps
        j = run_one(workload, extra, False, steps, args.warmup)
        lines.append(j)
        rows.append(fmt_row(label, "cold (HBM-resident)" if big or not workload.startswith("prefill") else "warm", j)
                    if not both else fmt_row(label, "warm", j))
        if both:
            j = run_one(workload, extra, True, steps, args.warmup)
            lines.append(j)
            rows.append(fmt_row("", j["config"]["cache"], j))
    head = ["| workload | cache | step us | tokens/s | dominant kernel us | roofline (kernel) | CPU oracle, whole step | "
            "parity max-abs / max-rel |", "|---|---|---|---|---|---|---|---|"]
    text = "\n".join(head + rows) + "\n"
    print(text)
    if args.out:
        with open(args.out, "w") as f:
            f.write(text)
    if args.json:
        with open(args.json, "w") as f:
            for j in lines:
                f.write(json.dumps(j) + "\n")


if __name__ == "__main__":
    main()
