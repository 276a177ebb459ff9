#!/usr/bin/env python3
"""Benchmark of the paged-KV attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input: paged_kv_append of the step's
new tokens, then paged attention over the paged cache (split-KV kernel + LSE merge for decode).  The
headline workload is the long-context decode (batch 16 x 131072 context, 64 query / 8 KV heads,
head_dim 128, bf16, page size 16); --workload selects the others.  Inputs are resident in HBM before
the timed region starts.  One JSON line is printed on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published

# HBM bytes per launch of the dominant kernel, measured once per workload with two rocprofv3 --pmc runs
# (FETCH_SIZE, WRITE_SIZE) and scaled by what the same counters read for the plain gather copy of known size
# (FETCH_SIZE x1.998, WRITE_SIZE x1.000); the summaries are under profiles/.
MEASURED_TRAFFIC = {
    "decode_b16_ctx131072_p16": {"read_bytes": 8588269000, "write_bytes": 9568500,
                                 "source": "profiles/decode_b16_ctx131072_p16.md"},
    "prefill_b4_s2048_causal": {"read_bytes": 154348000, "write_bytes": 67200000,
                                "source": "profiles/prefill_b4_s2048_causal.md"},
}

WORKLOADS = {
    # name: (config number, page size, context override)
    "decode_b16_ctx131072_p16": (5, 16, None),
    "decode_b16_ctx131072_p64": (5, 64, None),
    "decode_mixed64_shared_prefix": (4, 16, None),
    "decode_b8_ctx2048": (2, 16, 2048),
    "decode_b8_ctx1024": (2, 16, 1024),
    "decode_b8_ctx512": (2, 16, 512),
    "decode_b8_ctx256": (2, 16, 256),
    "decode_b8_ctx128": (2, 16, 128),
    "decode_fp32_single": (1, 16, None),
    "prefill_b4_s2048_causal": (3, 16, None),
    # jagged batches through the prefill entry point
    "prefill_chunk1024_on_ctx31744": (6, 16, None),
    "mixed_60_decode_4_prefill512": (7, 16, None),
    "speculative_4_tokens_b64_mixed": (8, 16, None),
    # the paper's own setting (Sec. IV): one LLaMA-7B layer (32 heads, no grouping, head_dim 128, fp16), 64-token pages,
    # one sequence; a decode step at the two ends of its 128 ... 2048-token range and the longest prompt's prefill
    "paper_llama7b_decode_ctx128": (9, 64, 128),
    "paper_llama7b_decode_ctx2048": (9, 64, 2048),
    "paper_llama7b_prefill_s2048": (10, 64, 2048),
    # plain paged copy of known size (Algorithm 1 Gather over 16 x 65536 tokens): calibrates HBM byte counters
    "gather_copy_calibration": (5, 16, 65536),
    # plain contiguous read of as many bytes as the 16 x 131072 decode step streams (2 x 4 GiB): the rate the memory
    # system gives the simplest reader, the yardstick for the decode kernel's fraction of the 8 TB/s peak
    "contiguous_read_calibration": (5, 16, None),
    # host-side KV page manager under serving churn (Algorithm 1 Reserve; Sec. III-B): not an attention workload
    "page_manager_serving": (None, 16, None),
}


def measured_traffic(args):
    """The committed counter figures belong to a workload as it is defined; a run that overrides its shape, element
    type or hooks has no measured traffic."""
    if args.head_dim or args.page_size or args.window or args.alibi or args.dtype == "fp16" or args.heads:
        return None
    return MEASURED_TRAFFIC.get(args.workload)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="decode_b16_ctx131072_p16", choices=sorted(WORKLOADS))
    ap.add_argument("--no-oracle", action="store_true", help="skip the CPU-oracle baseline / parity leg")
    ap.add_argument("--no-prefill", action="store_true", help="skip the extra measurements of the default run (prefill workload, other configurations)")
    ap.add_argument("--oracle-seqs", type=int, default=12, help="sequences of the workload the oracle is timed on")
    ap.add_argument("--dtype", choices=["default", "bf16", "fp16"], default="default",
                    help="16-bit element type of the pools (fp16 is the paper's own precision)")
    ap.add_argument("--page-size", type=int, default=0, help="override the workload's page size (power of two)")
    ap.add_argument("--head-dim", type=int, default=0, choices=[0, 64, 128, 256],
                    help="override the head_dim of the 16-bit workloads (default 128)")
    ap.add_argument("--heads", default="", help="HQ,HKV: override the 64 / 8 heads of the decode_b16_ctx131072 workloads "
                                                "(e.g. 8,1: one shard of an 8-way tensor-parallel model)")
    ap.add_argument("--window", type=int, default=0, help="sliding window in tokens (0 = off)")
    ap.add_argument("--alibi", action="store_true", help="add a linear position bias per head")
    ap.add_argument("--cold", action="store_true",
                    help="small decode workloads: rotate through copies of the pools (>= 512 MB in total) so that "
                         "every step misses the 256 MB last-level cache; default is warm (one pool)")
    ap.add_argument("--step", choices=["fused", "pair"], default="fused",
                    help="decode workloads: one paged_decode_step call per step (the append happens inside; default) "
                         "or the pair paged_kv_append + paged_attention_decode")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="library option set through pa_set_option before the run (repeatable), e.g. decode_short=-1")
    ap.add_argument("--launch", choices=["direct", "graph"], default="direct",
                    help="graph: capture one step (append + attention + merge) in a HIP graph and replay it; for the "
                         "small workloads, whose step is shorter than the host's launch overhead")
    return ap.parse_args()


STEP_STATS = {}


def time_steps(torch, step, steps, warmup, stats_key=None):
    """Average wall time of `steps` steps (barrier + synchronize on both sides).  With stats_key, events recorded
    between the steps on the launch stream also give the spread of the individual steps' GPU times."""
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)] if stats_key else None
    t0 = time.perf_counter()
    for i in range(steps):
        if marks:
            marks[i].record()
        step()
    if marks:
        marks[steps].record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    if marks:
        us = sorted(marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(steps))
        STEP_STATS[stats_key] = {"median_us": round(us[len(us) // 2], 2), "min_us": round(us[0], 2),
                                 "max_us": round(us[-1], 2), "note": "per-step GPU time between stream events"}
    return sec


def run_oracle_sample(sub, out_gpu_rows, mods=None):
    """Time the CPU oracle (append + attention) on whole sequences of the workload (host copies taken
    before the GPU path ran) and compare the GPU rows of those sequences with it."""
    import oracle
    from tests import parity
    t0 = time.perf_counter()
    _, _, ref, _ = parity.oracle_step(oracle, sub, mods=mods)
    dt = time.perf_counter() - t0
    got = parity.to_f64(out_gpu_rows)
    max_abs, max_rel = parity.errors(got, ref)
    import numpy as np
    unfloored = bool((np.abs(got - ref) <= 1e-2 + 2e-2 * np.abs(ref)).all())
    return dt, max_abs, max_rel, oracle.num_threads(), unfloored


def run_gather_calibration(torch, pa, binding, w, args):
    """Time paged_kv_gather, a pure copy: it reads and writes exactly sum(len) * 2*Hkv*d*E bytes."""
    import numpy as np
    cu = torch.tensor(np.concatenate([[0], np.cumsum(w.seq_lens_host)]), dtype=torch.int32, device=w.q.device)
    total = int(sum(w.seq_lens_host))

    def step():
        pa.paged_kv_gather(w.k_cache, w.v_cache, w.block_table, w.seq_lens, cu, total, w.max_seq_len)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.pa_profile_reset()
    binding.pa_profile_enable(True)
    sec = time_steps(torch, step, args.steps, 0)
    binding.pa_profile_enable(False)
    n, ms = binding.pa_profile_read("paged_kv_gather_kernel")
    nbytes = w.logical_kv_bytes()
    ach = nbytes / (ms / n * 1e-3) / 1e9
    print(json.dumps({
        "metric": "paged_gather_us_per_step", "value": round(sec * 1e6, 2), "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": args.workload, "tokens": total, "bytes_read": nbytes, "bytes_written": nbytes},
        "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None, "kernel": "paged_kv_gather_kernel",
                     "algorithmic_bytes": nbytes, "note": "achieved counts bytes read; as many are written"}}))


def run_read_calibration(torch, binding, w, args):
    """Time pa_stream_read over the first 4 GiB of each pool of the 16 x 131072 workload (8 589 934 592 bytes in all,
    the bytes one decode step of that workload streams)."""
    each = 4 << 30
    sink = torch.zeros(16, dtype=torch.uint8, device=w.q.device)

    def step():
        binding.pa_stream_read(w.k_cache, w.v_cache, each, sink)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.pa_profile_reset()
    binding.pa_profile_enable(True)
    time_steps(torch, step, args.steps, 0)
    binding.pa_profile_enable(False)
    n, ms = binding.pa_profile_read("pa_stream_read_kernel")
    sec = time_steps(torch, step, args.steps, 0)
    ach = 2 * each / (ms / n * 1e-3) / 1e9
    print(json.dumps({
        "metric": "contiguous_read_us_per_step", "value": round(sec * 1e6, 2), "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "u8", "data": "synthetic",
        "config": {"workload": args.workload, "bytes_read": 2 * each, "buffers": 2, "launch": "2048 workgroups x 512 "
                   "threads, 16 bytes per lane, 8 loads in flight per lane"},
        "kernels": {"pa_stream_read_kernel": {"launches": n, "avg_us": ms * 1e3 / n}},
        "roofline": {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": None, "kernel": "pa_stream_read_kernel",
                     "algorithmic_bytes": 2 * each}}))


def run_other_configs(torch, pa, binding, W, dev):
    """The other decode configurations and the plain-read yardstick, briefly, for the default run's line: step time
    (30 steps without events), the dominant kernel's time (30 steps with the library's events) and its fraction of
    the HBM peak.  No oracle leg here: `bench_all.py` has every configuration with oracle time and parity."""
    res = {}
    names = ["decode_fp32_single", "decode_b8_ctx128", "decode_b8_ctx256", "decode_b8_ctx512", "decode_b8_ctx1024",
             "decode_b8_ctx2048", "decode_mixed64_shared_prefix"]
    for wl in names:
        cfg, P, ctx = WORKLOADS[wl]
        w = W.config(cfg, device=dev, page_size=P, context=ctx, poison=False)
        ws = torch.empty(pa.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.total_q,
                                                            w.max_seq_len), dtype=torch.uint8, device=dev)
        out = torch.empty_like(w.q)
        step = pa.prepare_decode_step(w.k_cache, w.v_cache, w.k_new, w.v_new, w.q, w.block_table, w.seq_lens,
                                      w.max_seq_len, w.scale, out=out, workspace=ws)
        binding.pa_profile_enable(True)
        for _ in range(10):
            step()
        torch.cuda.synchronize()
        binding.pa_profile_reset()
        time_steps(torch, step, 30, 0)
        binding.pa_profile_enable(False)
        sec = time_steps(torch, step, 30, 0)
        dom = None
        for name in ("paged_decode_mfma_kernel", "paged_decode_short_kernel", "paged_attention_generic_kernel"):
            n, ms = binding.pa_profile_read(name)
            if n:
                dom = (name, ms * 1e3 / n)
                break
        binding.pa_profile_reset()
        nbytes = w.logical_kv_bytes()
        res[wl] = {"us_per_step": round(sec * 1e6, 2), "tokens_per_s": round(w.total_q / sec, 1), "kernel": dom[0],
                   "kernel_avg_us": round(dom[1], 2), "kv_bytes_per_step": nbytes,
                   "cache": "warm (fits the 256 MB last-level cache)" if nbytes < (200 << 20) else "HBM-resident",
                   "hbm_frac_kernel": round(nbytes / (dom[1] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
        del w, ws, out, step
        torch.cuda.empty_cache()
    each = 4 << 30
    a, b = (torch.empty(each, dtype=torch.uint8, device=dev) for _ in range(2))
    sink = torch.zeros(16, dtype=torch.uint8, device=dev)

    def read():
        binding.pa_stream_read(a, b, each, sink)
    for _ in range(3):
        read()
    torch.cuda.synchronize()
    binding.pa_profile_reset()
    binding.pa_profile_enable(True)
    time_steps(torch, read, 10, 0)
    binding.pa_profile_enable(False)
    n, ms = binding.pa_profile_read("pa_stream_read_kernel")
    binding.pa_profile_reset()
    res["contiguous_read_calibration"] = {"kernel": "pa_stream_read_kernel", "kernel_avg_us": round(ms * 1e3 / n, 1),
                                          "bytes": 2 * each,
                                          "hbm_frac_kernel": round(2 * each / (ms / n * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)}
    return res


def run_page_manager(torch, binding, args, P):
    """Serving churn through pa_pool_*: 256 live sequences grow by one token per step (one page pop every P
    steps per sequence, its row entry copied to the device table on the stream); every step four sequences end
    (release) and four prompts of 64..2048 tokens are admitted (reserve).  Times host calls only: they are what
    the manager costs per step; a step is args.steps iterations of the whole batch."""
    import random
    B, max_blocks, pages = 256, 512, 256 * 160
    table = torch.zeros((B, max_blocks), dtype=torch.int32, device="cuda:0")
    pool = binding.pa_pool_create(pages, P, B, max_blocks, table)
    rng = random.Random(7)
    lens = [rng.randrange(64, 2048) for _ in range(B)]
    for s in range(B):
        binding.pa_pool_reserve(pool, s, lens[s])
    lib = binding.load_library()
    import ctypes
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    i32 = ctypes.c_int32
    n_calls = pops = 0

    def step():
        nonlocal n_calls, pops
        for s in range(B):
            lens[s] = min(lens[s] + 1, max_blocks * P)
            pops += lens[s] % P == 1
            assert lib.pa_pool_reserve(pool, i32(s), i32(lens[s]), stream) == 0
        for _ in range(4):
            s = rng.randrange(B)
            assert lib.pa_pool_release(pool, i32(s), stream) == 0
            lens[s] = rng.randrange(64, 2048)
            assert lib.pa_pool_reserve(pool, i32(s), i32(lens[s]), stream) == 0
        n_calls += B + 8

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    n_calls = pops = 0
    sec = time_steps(torch, step, args.steps, 0)
    # the same calls on a pool without a device table: the bookkeeping alone
    host = binding.pa_pool_create(pages, P, B, max_blocks)
    null = ctypes.c_void_p(0)
    t0 = time.perf_counter()
    reps = 200000
    for i in range(reps):
        lib.pa_pool_reserve(host, i32(0), i32((i % 4096) + 1), null)
        if i % 4096 == 4095:
            lib.pa_pool_release(host, i32(0), null)
    per_call_host = (time.perf_counter() - t0) / reps
    binding.pa_pool_destroy(host)
    binding.pa_pool_destroy(pool)
    print(json.dumps({
        "metric": "page_manager_us_per_serving_step", "value": round(sec * 1e6, 2), "unit": "us/step", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 5), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "int32", "data": "synthetic",
        "config": {"workload": args.workload, "live_sequences": B, "page_size": P, "pages": pages,
                   "calls_per_step": n_calls // args.steps, "page_pops_per_step": round(pops / args.steps, 1)},
        "host_us_per_call_with_device_table": round(sec * 1e6 / (n_calls / args.steps), 3),
        "host_us_per_call_bookkeeping_only": round(per_call_host * 1e6, 3),
        "note": "both per-call figures include the Python ctypes call (about 0.3-0.5 us)"}))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: every box of this build has one, and the path has no multi-GPU part "
              f"(--gpus {args.gpus} refused).", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2506_07311_amd as pa
    from paper_2506_07311_amd import binding, workloads as W

    pa.load_library()
    for item in args.option:
        name, _, value = item.partition("=")
        binding.pa_set_option(name, int(value))
    dev = "cuda:0"
    cfg, P, ctx = WORKLOADS[args.workload]
    if args.workload == "page_manager_serving":
        return run_page_manager(torch, binding, args, P)
    if args.page_size:
        P = args.page_size
    heads = tuple(int(x) for x in args.heads.split(",")) if args.heads else None
    w = W.config(cfg, device=dev, page_size=P, context=ctx, poison=True, head_dim=args.head_dim or None, heads=heads)
    if args.dtype == "fp16" and w.dtype == torch.bfloat16:
        # the same N(0,1) draws rounded to fp16 instead of bf16 (NaN poison survives the conversion)
        for name in ("k_cache", "v_cache", "q", "k_new", "v_new"):
            setattr(w, name, getattr(w, name).to(torch.float16))
        w.dtype = torch.float16
    mods = {}
    if args.window:
        mods["window"] = args.window
    if args.alibi:
        mods["alibi_slopes"] = torch.tensor([2.0 ** (-8.0 * (h + 1) / w.num_q_heads) for h in range(w.num_q_heads)],
                                            dtype=torch.float32, device=dev)
    torch.cuda.synchronize()
    is_prefill = cfg in (3, 6, 7, 8, 10)
    if args.workload == "gather_copy_calibration":
        return run_gather_calibration(torch, pa, binding, w, args)
    if args.workload == "contiguous_read_calibration":
        return run_read_calibration(torch, binding, w, args)
    seqs = list(range(min(args.oracle_seqs, w.batch)))
    sub = None if args.no_oracle else W.restrict(w, seqs, device="cpu")

    ws = torch.empty(pa.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.total_q, w.max_seq_len),
                     dtype=torch.uint8, device=dev)
    out = torch.empty_like(w.q)

    # cold runs: as many copies of the two pools as it takes to exceed 512 MB, used round-robin
    # (the queries rotate with them: a prefill's Q is as large as its K)
    pools = [(w.k_cache, w.v_cache, w.q)]
    if args.cold:
        per_copy = 2 * w.k_cache.numel() * w.k_cache.element_size()
        while len(pools) * per_copy < (512 << 20) and len(pools) < 256:
            pools.append((w.k_cache.clone(), w.v_cache.clone(), w.q.clone()))
    # One step = append + attention (+ merge).  The arguments of the two calls are marshalled once per pool copy
    # (binding.prepare_*): the small workloads' steps are shorter on the GPU than converting the arguments again.
    fused = args.step == "fused" and not is_prefill and w.k_new.shape[0] == w.batch

    def make_step(kc, vc, qq):
        if fused:   # one new token per sequence at its last position, then decode: one call
            return pa.prepare_decode_step(kc, vc, w.k_new, w.v_new, qq, w.block_table, w.seq_lens, w.max_seq_len,
                                          w.scale, out=out, workspace=ws, **mods)
        app = pa.prepare_kv_append(kc, vc, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table)
        if is_prefill and mods:
            return lambda: (app(), pa.paged_attention_prefill_mod(kc, vc, qq, w.cu_q_lens, w.max_q_len, w.block_table,
                                                                 w.seq_lens, w.max_seq_len, w.scale, w.causal, out=out,
                                                                 workspace=ws, **mods))
        if is_prefill:
            att = pa.prepare_prefill(kc, vc, qq, w.cu_q_lens, w.max_q_len, w.block_table, w.seq_lens, w.max_seq_len,
                                     w.scale, w.causal, out=out, workspace=ws)
        elif mods:
            return lambda: (app(), pa.paged_attention_decode_mod(kc, vc, qq, w.block_table, w.seq_lens, w.max_seq_len,
                                                                w.scale, out=out, workspace=ws, **mods))
        else:
            att = pa.prepare_decode(kc, vc, qq, w.block_table, w.seq_lens, w.max_seq_len, w.scale, out=out,
                                    workspace=ws)
        return lambda: (app(), att())

    steps_by_pool = [make_step(*p) for p in pools]
    turn = [0]

    def step():
        steps_by_pool[turn[0] % len(steps_by_pool)]()
        turn[0] += 1

    # timed region: per-kernel HIP events (recorded by the library on the launch stream) stay on, so the
    # dominant kernel's duration comes from the same K steps the step time does
    # the warm-up runs with the per-kernel events on as well, so that the timed region reuses their event objects
    binding.pa_profile_enable(True)
    for _ in range(max(args.warmup, min(args.steps, 3))):
        step()
    binding.pa_profile_enable(False)
    torch.cuda.synchronize()
    binding.pa_profile_reset()
    kernels = {}
    if args.launch == "graph":
        # per-kernel events cannot be recorded inside a captured graph: time them in K direct steps first,
        # then time the step itself as K replays of the captured graph
        binding.pa_profile_enable(True)
        time_steps(torch, step, args.steps, 0)
        binding.pa_profile_enable(False)
        # (prepared calls carry the stream they were prepared on: the captured step is prepared on the capture stream)
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            captured = make_step(*pools[0])
            captured()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                captured()
        torch.cuda.synchronize()
        out.zero_()
        torch.cuda.synchronize()
        sec = time_steps(torch, graph.replay, args.steps, 2)
        if not bool(out.any().item()):
            raise SystemExit("bench.py: the captured graph did not run the step (output untouched)")
    else:
        # Two passes over the same K steps: one with the library's per-kernel events on the launch stream (the
        # kernels' durations), one without them (the step time: six event records per step cost 20-30 us of stream
        # time, which is 2 % of the longest step here and more than the whole of the shortest).
        binding.pa_profile_enable(True)
        sec_events = time_steps(torch, step, args.steps, 0)
        binding.pa_profile_enable(False)
        sec = time_steps(torch, step, args.steps, 0)
        time_steps(torch, step, args.steps, 0, stats_key="step")    # spread of the single steps (one event between steps)
        kernel_timing = ("per-kernel events in a pass of their own over the same K steps "
                         f"({sec_events * 1e6:.1f} us per step with them); step time from the pass without them")
    for name in ("paged_kv_append_kernel", "paged_kv_append_last_kernel", "paged_decode_mfma_kernel",
                 "paged_decode_short_kernel",
                 "paged_attention_generic_kernel",
                 "paged_attention_merge_kernel", "paged_prefill_mfma_kernel"):
        n, ms = binding.pa_profile_read(name)
        if n:
            kernels[name] = {"launches": n, "avg_us": ms * 1e3 / n}
    binding.pa_profile_reset()

    us = sec * 1e6
    kv_bytes = w.logical_kv_bytes()
    if args.window and not is_prefill:   # only the window is read
        kv_bytes = sum(min(L, args.window) for L in w.seq_lens_host) * 2 * w.num_kv_heads * w.head_dim * 2
    tokens = w.total_q                      # tokens produced (decode) / processed (prefill) per step
    result = {
        "metric": "paged_prefill_us_per_step" if is_prefill else "paged_decode_us_per_step",
        "value": round(us, 2), "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us / 1e3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": {torch.bfloat16: "bf16", torch.float16: "f16", torch.float32: "f32"}[w.dtype], "data": "synthetic",
        "config": {"workload": args.workload, "batch": w.batch, "context": w.max_seq_len,
                   "num_q_heads": w.num_q_heads, "num_kv_heads": w.num_kv_heads, "head_dim": w.head_dim,
                   "page_size": w.page_size, "pool_pages": w.num_pages,
                   "step": "paged_decode_step: append + attention (+ merge) in one call" if fused
                   else "append + attention (+ merge)",
                   **({"options": args.option} if args.option else {}),
                   "launch": args.launch, "cache": f"cold ({len(pools)} pool copies)" if args.cold else "warm",
                   **({"window": args.window} if args.window else {}),
                   **({"alibi": True} if args.alibi else {})},
        "tokens_per_s": round(tokens / sec, 1),
        "kv_bytes_per_step": kv_bytes,
        "step_hbm_gbps": round(kv_bytes / sec / 1e9, 1),
        "step_hbm_frac": round(kv_bytes / sec / 1e9 / HBM_PEAK_GBPS, 4),
        "kernels": kernels,
    }
    if args.launch != "graph":
        result["kernel_timing"] = kernel_timing
        result["us_per_step_with_kernel_events"] = round(sec_events * 1e6, 2)
    if "step" in STEP_STATS:
        result["step_us_stats"] = STEP_STATS["step"]
    G = w.num_q_heads // w.num_kv_heads
    # in a prefill call, sequences with q_len * G <= 16 are computed by the decode kernel (bound: their KV bytes),
    # the others by the prefill kernel (bound: their flops)
    small = [ql * G <= 16 for ql in w.q_lens_host]
    t_dec = kernels.get("paged_decode_mfma_kernel", {}).get("avg_us", 0.0)
    t_pre = max(kernels.get("paged_prefill_mfma_kernel", {}).get("avg_us", 0.0),
                kernels.get("paged_attention_generic_kernel", {}).get("avg_us", 0.0))
    if is_prefill and t_dec > t_pre:
        small_bytes = sum(L for L, sm in zip(w.seq_lens_host, small) if sm) * 2 * w.num_kv_heads * w.head_dim * 2
        ach = small_bytes / (t_dec * 1e-6) / 1e9
        result["roofline"] = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(args),
                              "kernel": "paged_decode_mfma_kernel", "algorithmic_bytes": small_bytes,
                              "note": "KV bytes of the sequences the decode kernel computes in this call"}
    elif is_prefill:
        routed = "paged_decode_mfma_kernel" in kernels
        def pairs(ql, L):
            # (query, visible key) pairs of one head
            if not args.window:
                return ql * (L - ql) + ql * (ql + 1) // 2 if w.causal else ql * L
            n = 0
            for i in range(ql):
                pos = L - ql + i
                lo, hi = max(0, pos - args.window + 1), (pos + 1 if w.causal else min(L, pos + args.window))
                n += hi - lo
            return n
        flops = sum(4 * w.num_q_heads * w.head_dim * pairs(ql, L)
                    for ql, L, sm in zip(w.q_lens_host, w.seq_lens_host, small) if not (sm and routed))
        dom = kernels.get("paged_prefill_mfma_kernel") or kernels.get("paged_attention_generic_kernel")
        ach = flops / (dom["avg_us"] * 1e-6) / 1e12
        result["roofline"] = {"bound": "mfma", "achieved": round(ach, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                              "unit": "TFLOP/s", "frac": round(ach / MFMA_BF16_PEAK_TFLOPS, 4),
                              "traffic": measured_traffic(args),
                              "kernel": "paged_prefill_mfma_kernel" if "paged_prefill_mfma_kernel" in kernels
                              else "paged_attention_generic_kernel", "useful_flops": flops}
    else:
        name = next(n for n in ("paged_decode_mfma_kernel", "paged_decode_short_kernel",
                                "paged_attention_generic_kernel") if n in kernels)
        ach = kv_bytes / (kernels[name]["avg_us"] * 1e-6) / 1e9
        result["roofline"] = {"bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                              "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": measured_traffic(args),
                              "kernel": name,
                              "algorithmic_bytes": kv_bytes}

    if not args.no_oracle:
        cu = w.cu_q_lens.cpu().tolist()
        rows = [r for s_ in seqs for r in range(cu[s_], cu[s_ + 1])]
        omods = {k: (v.cpu().numpy() if hasattr(v, "cpu") else v) for k, v in mods.items()} or None
        dt, max_abs, max_rel, cores, unfloored = run_oracle_sample(sub, out[rows], omods)
        scale_up = w.batch / len(seqs)
        result["cpu_baseline"] = {"value": round(dt * scale_up * 1e6, 1), "unit": "us/step", "cores": cores,
                                  "kind": "oracle",
                                  "sample": f"{len(seqs)} of {w.batch} sequences (all heads, full context) in "
                                            f"{dt:.2f} s, scaled x{scale_up:g}"}
        result["parity_sample"] = {"max_abs": max_abs, "max_rel_rms_floored": max_rel,
                                   "within_1e-2_plus_2e-2_of_ref_elementwise": unfloored, "sequences": seqs}

    if not is_prefill and not args.no_prefill:
        try:     # extras: a failure here must not cost the line of the workload that was asked for
            del w, ws, out
            torch.cuda.empty_cache()
            wp = W.config(3, device=dev, poison=False)
            wsp = torch.empty(pa.paged_attention_workspace_bytes(wp.batch, wp.num_q_heads, wp.head_dim, wp.total_q,
                                                                 wp.max_seq_len), dtype=torch.uint8, device=dev)
            outp = torch.empty_like(wp.q)

            p_app = pa.prepare_kv_append(wp.k_cache, wp.v_cache, wp.k_new, wp.v_new, wp.seq_ids, wp.positions,
                                         wp.block_table)
            p_att = pa.prepare_prefill(wp.k_cache, wp.v_cache, wp.q, wp.cu_q_lens, wp.max_q_len, wp.block_table,
                                       wp.seq_lens, wp.max_seq_len, wp.scale, wp.causal, out=outp, workspace=wsp)

            def pstep():     # arguments marshalled once, as in the prefill workload's own run
                p_app()
                p_att()
            for _ in range(max(20, args.warmup)):        # (the GPU has idled through the oracle's seconds on the host:
                pstep()                                  #  a few milliseconds of the workload bring its clock back)
            torch.cuda.synchronize()
            binding.pa_profile_reset()
            binding.pa_profile_enable(True)             # kernel durations: a pass with the per-kernel events ...
            time_steps(torch, pstep, max(30, args.steps), 0)
            binding.pa_profile_enable(False)
            psec = time_steps(torch, pstep, max(30, args.steps), 5)   # ... step time: the same steps without them
            S = wp.max_seq_len
            flops = 4 * wp.batch * wp.num_q_heads * wp.head_dim * S * (S + 1) // 2
            pk = None
            for name in ("paged_prefill_mfma_kernel", "paged_attention_generic_kernel"):
                n, ms = binding.pa_profile_read(name)
                if n:
                    pk = (name, ms * 1e3 / n)
                    break
            binding.pa_profile_reset()
            result["prefill"] = {"workload": "prefill_b4_s2048_causal", "us_per_step": round(psec * 1e6, 1),
                                 "tokens_per_s": round(wp.total_q / psec, 1), "kernel": pk[0],
                                 "kernel_avg_us": round(pk[1], 1), "useful_flops": flops,
                                 "mfma_tflops": round(flops / (pk[1] * 1e-6) / 1e12, 1),
                                 "mfma_frac": round(flops / (pk[1] * 1e-6) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
            if args.workload == "decode_b16_ctx131072_p16" and not args.option and not args.cold:
                del wp, wsp, outp, p_app, p_att
                torch.cuda.empty_cache()
                try:     # extras: a failure here must not cost the line of the workload that was asked for
                    result["other_configs"] = run_other_configs(torch, pa, binding, W, dev)
                except Exception as e:   # noqa: BLE001
                    result["other_configs"] = {"error": repr(e)[:300]}
        except Exception as e:   # noqa: BLE001
            result.setdefault("prefill", {"error": repr(e)[:300]})
    print(json.dumps(result))


if __name__ == "__main__":
    main()
