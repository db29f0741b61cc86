#!/usr/bin/env python3
"""Benchmark of the decode hot path (grow check, append, ragged attention, retire/refill) on ONE
MI355X, through the C ABI of libs3kv.so, on the synthetic workload C1 (GPT-J-shaped layer, batch 64,
128 consecutive decode steps: the configuration the headline metric is quoted on) unless --workload
says otherwise.

Prints ONE JSON line.  `value` is algorithmic bytes moved per second over the whole timed
region (all kernels, host bookkeeping included), inputs resident in HBM.  `roofline` is for the
dominant kernel (the attention kernel of the workload's cache type), timed with HIP events bound to
the kernel's own start and end, inside the same timed region.  `cpu_baseline` is the CPU oracle timed on this machine's host cores on a
bounded sample of the same workload.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed decode steps (default: per workload)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c1", choices=["c1", "c2", "c3", "c4", "c5", "c6"])
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--grid-blocks", type=int, default=0)
    ap.add_argument("--classes", type=int, default=0, help="length classes of the longest-first work order (0: library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not time the attention kernel with events")
    ap.add_argument("--event-every", type=int, default=16,
                    help="every k-th attention launch carries start/stop events (an evented launch costs a few us)")
    ap.add_argument("--c3-bytes", type=float, default=200e9)
    ap.add_argument("--heads", type=str, default="", help="c5 only: query heads, kv heads, head dim as Q,KV,D")
    ap.add_argument("--kv8", action="store_true", help="c5 only: e4m3 cache rows (bf16 queries) on top of the shared heads")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (not c3); the "
                    "default is the configuration the metric is quoted on")
    ap.add_argument("--unfused", action="store_true", help="append + attention + merge kernels instead of one")
    ap.add_argument("--drain", action="store_true", help="finished sequences are not replaced: the batch shrinks")
    ap.add_argument("--on-nomem", choices=("swap", "drop"), default="swap", help="a reservation that cannot be doubled: "
                    "swap = compaction or eviction to the host and later re-admission (the paper's supervisor; default), "
                    "drop = the sequence leaves the batch")
    ap.add_argument("--flush-mb", type=int, default=0, help="diagnostic: overwrite a buffer of this many MB between "
                    "steps so that the memory-side cache holds none of the previous step's rows; every launch is "
                    "then bracketed and only roofline.* is meaningful (value includes the flushes)")
    return ap.parse_args()


DEFAULT_STEPS = {"c1": (128, 8), "c2": (256, 8), "c3": (3, 1), "c4": (56, 8), "c5": (128, 8), "c6": (128, 8)}  # (timed, warm-up)


def make_device_sources(w, eng, torch, ring=8):
    """Inputs resident in HBM before the timed region: a ring of N(0,1) q/k/v tensors and a pool
    of prompt rows that newcomers are filled from.  Seeded torch generator on the device."""
    gen = torch.Generator(device=eng.dev)
    gen.manual_seed(w.seed)
    tdt = eng.act_dtype_torch()
    rows = torch.randn((2, w.max_len, w.kv_heads, w.head_dim), generator=gen, device=eng.dev, dtype=torch.float32)
    if eng.kv_dtype_torch() == torch.uint8:  # 8-bit cache rows: N(0,1) as e4m3 codes, converted by torch on the host
        rows = rows.cpu().to(torch.float8_e4m3fn).view(torch.uint8).to(eng.dev)
    else:
        rows = rows.to(tdt)
    state = {"i": 0, "qkv": None}

    def prefill(serial, layer, n_rows):
        return rows[0, :n_rows], rows[1, :n_rows]

    def tensors(layer, n):
        if state["qkv"] is None or state["qkv"].shape[2] < n:  # sized once, for the largest batch seen
            bmax = max(n, eng.n_active, 1 if w.arena_bytes else len(w.seqs))
            state["qkv"] = torch.randn((ring, 3, bmax, w.n_heads, w.head_dim), generator=gen, device=eng.dev,
                                       dtype=torch.float32).to(tdt)
            if w.kv_heads < w.n_heads:  # shared key/value heads: contiguous [n][kv_heads][D] rows of their own
                state["kv"] = torch.randn((ring, 2, bmax, w.kv_heads, w.head_dim), generator=gen, device=eng.dev,
                                          dtype=torch.float32).to(tdt)
        t = state["qkv"][state["i"] % ring]
        kv = state["kv"][state["i"] % ring] if w.kv_heads < w.n_heads else t[1:]
        state["i"] += 1
        return t[0, :n], kv[0, :n], kv[1, :n]

    return prefill, tensors, (state, rows)


def read_traffic(kernel, workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this
    same command, if there is one (bench.py cannot collect counters itself)."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return int(float(line.split(":")[1]))
    except OSError:
        pass
    return None


def cpu_baseline(w, lens, budget_s=12.0):
    """Time the oracle as it stands (fp32 attention, OpenMP over (sequence, head) on all host
    cores) on the batch state at the start of the timed region: whole-batch passes over one layer are repeated
    until the time budget is used (at least one pass; a pass that would not fit the budget is cut
    to a prefix of the batch).  K/V values are N(0,1) like the GPU's; the oracle's run time does
    not depend on them."""
    import numpy as np

    from oracle import kv_oracle as orc
    from paper_2306_06000_amd import workloads as wl

    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    omp = int(os.environ.get("OMP_NUM_THREADS", "0") or 0)
    if omp > 0:
        cores = min(cores, omp)
    H, D = w.n_heads, w.head_dim
    rng = np.random.default_rng(w.seed)
    kv = wl.normal_bits(rng, (2, int(w.max_len), w.kv_heads, D), w.dtype)
    done_bytes, done_seqs, t_used, used = 0, 0, 0.0, cores
    n_take = min(lens.size, 16)  # first a small probe to size the passes
    passes = 0
    while t_used < budget_s:
        idx = np.arange(n_take)
        q = wl.normal_bits(rng, (idx.size, H, D), w.q_dtype)
        t0 = time.perf_counter()
        _, used = orc.attention_ragged(q, [kv[0]] * idx.size, [kv[1]] * idx.size, lens[idx], w.dtype, None, "f32",
                                       threads=cores, q_dtype=w.q_dtype)
        dt = time.perf_counter() - t0
        t_used += dt
        done_bytes += int(2 * w.kv_heads * D * w.elem_bytes * lens[idx].sum() + idx.size * H * D * (2 + 4))
        done_seqs += int(idx.size)
        passes += 1
        rate = idx.size / dt
        n_take = int(max(1, min(lens.size, rate * min(budget_s - t_used, 4.0))))
        if budget_s - t_used < 0.05:
            break
    # the same code on one thread (plain serial loops), on a short prefix
    n1 = min(lens.size, 4)
    q1 = wl.normal_bits(rng, (n1, H, D), w.q_dtype)
    t0 = time.perf_counter()
    orc.attention_ragged(q1, [kv[0]] * n1, [kv[1]] * n1, lens[:n1], w.dtype, None, "f32", threads=1, q_dtype=w.q_dtype)
    dt1 = time.perf_counter() - t0
    one_thread = (2 * w.kv_heads * D * w.elem_bytes * int(lens[:n1].sum()) + n1 * H * D * (2 + 4)) / dt1 / 1e9
    return {"value": round(done_bytes / t_used / 1e9, 4), "unit": "GB/s", "cores": int(used), "kind": "oracle",
            "one_thread_value": round(one_thread, 4),
            "seq_steps_per_s": round(done_seqs / t_used, 2),
            "sample": f"one layer of oracle attention over prefixes of the batch state at the start of the timed region ({lens.size} sequences), "
                      f"{passes} passes, {done_seqs} sequence-steps, {t_used:.1f} s of CPU work, OpenMP over "
                      "(sequence, head)"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2306_06000_amd import binding as s3
    from paper_2306_06000_amd import workloads as wl
    from paper_2306_06000_amd.engine import DecodeEngine

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    s3.lib()
    kw = {"batch": args.batch} if args.batch > 0 else {}
    if args.heads and args.workload == "c5":
        hq, hkv, hd = (int(x) for x in args.heads.split(","))
        kw.update(n_heads=hq, n_kv_heads=hkv, head_dim=hd)
    if args.kv8 and args.workload == "c5":
        kw.update(dtype=wl.E4M3)
    w = {"c1": wl.c1, "c2": wl.c2, "c4": wl.c4, "c5": wl.c5, "c6": wl.c6}[args.workload](**kw) if args.workload != "c3" else wl.c3(
        target_bytes=int(args.c3_bytes))
    if args.drain:
        w.refill = False
    shared_kv = w.kv_heads < w.n_heads  # not one of the paper's models: measured as a widening, not the headline
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[args.workload][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[args.workload][1]
    eng = DecodeEngine(w, log_events=False, fused=not args.unfused, on_nomem=args.on_nomem)
    if args.variant >= 0:
        s3.check(s3.s3_kv_set_param(eng.arena, "variant", args.variant))
    if args.chunk:
        s3.check(s3.s3_kv_set_param(eng.arena, "chunk", args.chunk))
    if args.grid_blocks:
        s3.check(s3.s3_kv_set_param(eng.arena, "grid_blocks", args.grid_blocks))
    if args.classes:
        s3.check(s3.s3_kv_set_param(eng.arena, "classes", args.classes))
    prefill, tensors, _keep = make_device_sources(w, eng, torch)
    eng.start(prefill, stop_when_full=(args.workload == "c3"))
    torch.cuda.synchronize()

    for _ in range(warmup):
        eng.step(tensors, prefill)
    torch.cuda.synchronize()
    lens_at_start = eng.len.copy()
    every = 1 if args.flush_mb else max(1, args.event_every)
    flush = torch.empty(args.flush_mb << 20, dtype=torch.uint8, device=eng.dev) if args.flush_mb else None
    if not args.no_kernel_events:
        s3.check(s3.s3_kv_set_param(eng.arena, "profile", every))
    grown0, retired0 = eng.n_grown, eng.n_retired
    total_bytes, seq_steps, launch_bytes, steps_done = 0, 0, [], 0
    # The interpreter's cyclic garbage collector is kept out of the timed region (a full collection takes
    # tens of milliseconds here and would land on whichever step triggers it): collect now, resume after.
    gc.collect()
    gc.disable()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        if eng.n_active == 0:  # drain runs: every sequence has finished
            break
        if flush is not None:
            flush.fill_(1)
        eng.step(tensors, prefill)
        steps_done += 1
        total_bytes += eng.last_step_bytes
        seq_steps += eng.last_step_seqs
        launch_bytes += [eng.last_step_bytes // w.n_layers] * w.n_layers
    t_enqueue = time.perf_counter() - t0  # host time to enqueue every step (no device wait in it)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    gc.enable()
    args.steps, args.warmup = steps_done, warmup

    res = {
        "metric": "decode-attention achieved HBM GB/s (% of peak); sequence-steps/sec at batch B", "value": round(total_bytes / dt / 1e9, 2), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {0: "f16", 1: "bf16", 3: "e4m3 rows, 16-bit queries, f32 arithmetic"}[w.dtype], "data": "synthetic",
        "pct_of_peak_hbm": round(100 * total_bytes / dt / 1e9 / PEAK_HBM_GBPS, 2),
        "seq_steps_per_s": round(seq_steps / dt, 1),
        "host_enqueue_ms_per_step": round(t_enqueue / args.steps * 1e3, 5),
        "config": {"workload": w.name, "batch": int(lens_at_start.size), "n_layers": w.n_layers,
                   "n_heads": w.n_heads, "n_kv_heads": w.kv_heads, "head_dim": w.head_dim,
                   "mean_context_at_start": round(float(lens_at_start.mean()), 1),
                   "batch_at_end": int(eng.n_active), "refill": bool(w.refill),
                   "grows": eng.n_grown - grown0, "retired": eng.n_retired - retired0,
                   "swapped_out": eng.n_swapped_out, "swapped_in": eng.n_swapped_in, "compactions": eng.n_compactions,
                   "dropped": eng.n_evicted, "on_nomem": args.on_nomem,
                   "arena_GB": round(eng.arena_mem.numel() / 1e9, 3),
                   "algorithmic_GB_per_step": round(total_bytes / args.steps / 1e9, 4),
                   "path": "quantising append + shared-kv matrix-core attention over 8-bit rows + merge per layer" if shared_kv and w.dtype == 3 else
                           "shared-kv attention kernel (+ append launch for the vector-ALU kernel) + merge per layer" if shared_kv else
                           "one s3_decode_step kernel per layer (quantises and appends the new row, attends over 8-bit rows, merges)" if w.dtype == 3 else
                           "append+attention+merge kernels" if args.unfused else "one s3_decode_step kernel per layer",
                   "variant": s3.s3_kv_get_param(eng.arena, "variant")[1],
                   "chunk": s3.s3_kv_get_param(eng.arena, "chunk")[1]},
    }
    if not args.no_kernel_events:
        launches = s3.s3_kv_get_param(eng.arena, "profile_launches")[1]
        part_ns = s3.s3_kv_get_param(eng.arena, "profile_partial_ns")[1]
        merge_ns = s3.s3_kv_get_param(eng.arena, "profile_merge_ns")[1]
        sampled = launch_bytes[::every]  # the launches that were bracketed: every k-th, from the first
        assert len(sampled) == launches, (len(sampled), launches)
        per_launch_bytes = sum(sampled) / max(launches, 1)
        avg_us = part_ns / max(launches, 1) / 1e3
        achieved = per_launch_bytes / (avg_us * 1e-6) / 1e9 if avg_us > 0 else 0.0
        kind = s3.s3_kv_get_param(eng.arena, "kernel_kind")[1]
        kernel = {1: "attn_gqa_kernel", 2: "attn_gqa_mfma_kernel", 3: "attn_fp8_kernel", 4: "attn_gqa_mfma_kernel"}.get(
            kind, "attn_partial_kernel" if args.unfused else "attn_step_kernel")
        res["roofline"] = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1),
                           "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBPS, 4),
                           "traffic": read_traffic(kernel, args.workload), "avg_kernel_us": round(avg_us, 2),
                           "kernel_us_p10_p50_p90": [round(s3.s3_kv_get_param(eng.arena, f"profile_p{q}_ns")[1] / 1e3, 2)
                                                     for q in (10, 50, 90)],
                           "timed_launches": launches, "of_launches": len(launch_bytes),
                           "algorithmic_bytes_per_launch": int(per_launch_bytes)}
        if args.unfused:
            res["roofline"]["avg_merge_kernel_us"] = round(merge_ns / max(launches, 1) / 1e3, 2)
    if args.flush_mb:
        res["config"]["cache_flush_MB_between_steps"] = args.flush_mb
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(w, lens_at_start)
    eng.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
