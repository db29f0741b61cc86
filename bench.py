#!/usr/bin/env python3
"""Benchmark of the decode hot path (grow check, append, ragged attention, retire/refill) on ONE
MI355X, through the C ABI of libs3kv.so, on the synthetic workloads C1-C4.

With no --workload the four target workloads run in one process: C3 (28 GPT-J layers, 200 GB arena: the
largest single-GPU configuration) is the headline of the JSON line, C1, C2 and C4 follow in `per_config`.
--workload c1..c6 runs one workload only (profiling, sweeps, the shared-head and 8-bit variants).

Per workload: the arena is filled, the device is brought to its working clocks by the library's streaming
probe (which also says what a plain read reaches on this device), W warm-up steps, then
  pass 1  K timed steps, nothing but the product path: `value` = algorithmic bytes / wall time of the whole
          region (all kernels and the host bookkeeping), inputs resident in HBM;
  pass 2  the next K steps of the same run with EVERY attention launch bracketed by HIP events bound to the
          kernel's own start and end on the launch stream: `roofline` (average kernel duration, algorithmic
          bytes of exactly those launches).  Bracketing separates the dispatches and costs the host a few
          microseconds per launch, which is why it is kept out of pass 1.
`cpu_baseline` is the CPU oracle timed on this machine's host cores on a bounded sample of the same workload.
Prints ONE JSON line.
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
TARGETS = ("c3", "c1", "c2", "c4")  # headline first
METRIC = "decode-attention achieved HBM GB/s (% of peak); sequence-steps/sec at batch B"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed decode steps per workload (default: per workload)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="all", choices=["all", "c1", "c2", "c3", "c4", "c5", "c6"])
    ap.add_argument("--variant", type=int, default=-1)
    ap.add_argument("--chunk", type=int, default=0)
    ap.add_argument("--grid-blocks", type=int, default=0)
    ap.add_argument("--classes", type=int, default=0, help="length classes of the longest-first work order (0: library default)")
    ap.add_argument("--merge-sync", type=int, default=0, help="1: fence-ordered merge of chunks inside a launch")
    ap.add_argument("--gqa-merge", type=int, default=-1, help="shared heads, matrix-core kernel: 1 = chunks merge inside "
                    "the attention launch, 0 = merge launch (-1: library default)")
    ap.add_argument("--gqa-stream", type=int, default=-1, help="shared heads, matrix-core kernel: K rows read with the "
                    "streaming hint (1), with plain loads (0), by launch size (-1, the library's default)")
    ap.add_argument("--gqa-dynamic", type=int, default=-1, help="shared heads, matrix-core kernel: per cent of the work "
                    "list dealt by stride before waves claim positions (0 or -1, the default: all by stride)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-events", action="store_true", help="skip pass 2 (no events anywhere: for counter runs)")
    ap.add_argument("--c3-bytes", type=float, default=200e9)
    ap.add_argument("--heads", type=str, default="", help="c5 only: query heads, kv heads, head dim as Q,KV,D")
    ap.add_argument("--kv8", action="store_true", help="c5 only: e4m3 cache rows (bf16 queries) on top of the shared heads")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's batch size (not c3)")
    ap.add_argument("--unfused", action="store_true", help="append + attention + merge kernels instead of one")
    ap.add_argument("--drain", action="store_true", help="finished sequences are not replaced: the batch shrinks")
    ap.add_argument("--on-nomem", choices=("swap", "drop"), default="swap", help="a reservation that cannot be doubled: "
                    "swap = compaction or eviction to the host and later re-admission (the paper's supervisor; default), "
                    "drop = the sequence leaves the batch")
    ap.add_argument("--flush-mb", type=int, default=0, help="diagnostic: overwrite a buffer of this many MB between "
                    "steps so that the memory-side cache holds none of the previous step's rows (pass 2 only matters)")
    return ap.parse_args()


DEFAULT_STEPS = {"c1": (128, 8), "c2": (256, 8), "c3": (8, 2), "c4": (24, 8), "c5": (128, 8), "c6": (128, 8)}  # (timed, warm-up)


class DeviceSources:
    """Inputs resident in HBM before any timed region: a pool of prompt rows that newcomers are filled from and
    a ring of N(0,1) q / k_new / v_new sets, handed to the engine as raw device addresses (a step then costs
    the host no tensor indexing).  Seeded torch generator on the device."""

    def __init__(self, w, eng, torch, ring=8):
        self.w, self.eng, self.torch, self.ring = w, eng, torch, ring
        self.gen = torch.Generator(device=eng.dev)
        self.gen.manual_seed(w.seed)
        tdt = eng.act_dtype_torch()
        rows = torch.randn((2, w.max_len, w.kv_heads, w.head_dim), generator=self.gen, device=eng.dev, dtype=torch.float32)
        if eng.kv_dtype_torch() == torch.uint8:  # 8-bit cache rows: N(0,1) as e4m3 codes, converted by torch on the host
            rows = rows.cpu().to(torch.float8_e4m3fn).view(torch.uint8).to(eng.dev)
        else:
            rows = rows.to(tdt)
        self.rows = rows
        self.k_rows, self.v_rows = rows[0].data_ptr(), rows[1].data_ptr()
        self.i = 0
        self.q_ptr = self.k_ptr = self.v_ptr = None

    def prefill(self, serial, layer, n_rows):
        return self.k_rows, self.v_rows  # the first n_rows rows of the pool

    def size_for(self, bmax):
        """The q / k / v ring, once the batch is known: [ring][3][bmax][H][D]; a batch of n <= bmax uses the
        first n rows of a set, which are contiguous."""
        w, torch = self.w, self.torch
        tdt = self.eng.act_dtype_torch()
        self.qkv = torch.randn((self.ring, 3, bmax, w.n_heads, w.head_dim), generator=self.gen, device=self.eng.dev,
                               dtype=torch.float32).to(tdt)
        self.q_ptr = [self.qkv[r, 0].data_ptr() for r in range(self.ring)]
        if w.kv_heads < w.n_heads:  # shared key/value heads: contiguous [n][kv_heads][D] rows of their own
            self.kv = torch.randn((self.ring, 2, bmax, w.kv_heads, w.head_dim), generator=self.gen, device=self.eng.dev,
                                  dtype=torch.float32).to(tdt)
            self.k_ptr = [self.kv[r, 0].data_ptr() for r in range(self.ring)]
            self.v_ptr = [self.kv[r, 1].data_ptr() for r in range(self.ring)]
        else:
            self.k_ptr = [self.qkv[r, 1].data_ptr() for r in range(self.ring)]
            self.v_ptr = [self.qkv[r, 2].data_ptr() for r in range(self.ring)]

    def tensors(self, layer, n):
        r = self.i % self.ring
        self.i += 1
        return self.q_ptr[r], self.k_ptr[r], self.v_ptr[r]


def read_traffic(kernel, workload):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary of this
    workload (bench.py cannot collect counters itself), with the algorithmic bytes per launch of THAT run, so
    that the ratio compares one run with itself."""
    path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.txt")
    got = {}
    try:
        for line in open(path):
            for key in ("traffic_bytes_per_launch", "algorithmic_bytes_per_launch"):
                if line.startswith(key + ":"):
                    got[key] = int(float(line.split(":")[1]))
    except OSError:
        pass
    return got.get("traffic_bytes_per_launch"), got.get("algorithmic_bytes_per_launch")


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


def make_workload(name, args):
    from paper_2306_06000_amd import workloads as wl

    kw = {"batch": args.batch} if args.batch > 0 and name != "c3" else {}
    if args.heads and name == "c5":
        hq, hkv, hd = (int(x) for x in args.heads.split(","))
        kw.update(n_heads=hq, n_kv_heads=hkv, head_dim=hd)
    if args.kv8 and name == "c5":
        kw.update(dtype=wl.E4M3)
    w = wl.c3(target_bytes=int(args.c3_bytes)) if name == "c3" else {"c1": wl.c1, "c2": wl.c2, "c4": wl.c4, "c5": wl.c5,
                                                                     "c6": wl.c6}[name](**kw)
    if args.drain:
        w.refill = False
    return w


def prime_code_paths(torch):
    """Every kernel and every host path of a decode loop (doubling, retiring, refilling, batch patches, an
    eviction and its reload) is run once on a throw-away arena of a few hundred tokens before anything is timed:
    the first use of a path costs hundreds of microseconds (code loading, pinned staging memory), which would
    otherwise land on whichever timed step meets it first."""
    from paper_2306_06000_amd import workloads as wl
    from paper_2306_06000_amd.engine import DecodeEngine

    seqs = [wl.Seq(prompt=10 + 3 * i, output=3 + i % 5, predicted=14 + 3 * i) for i in range(6)]
    seqs[1] = wl.Seq(prompt=60, output=12, predicted=61)     # outgrows its slot: doubling
    seqs[2] = wl.Seq(prompt=120, output=12, predicted=121)   # outgrows it when nothing is free: swap
    pool = [wl.Seq(prompt=5 + i, output=4, predicted=9 + i) for i in range(8)]
    w = wl.Workload("prime", 99, 2, 16, 256, wl.F16, 64, 512, len(seqs), 16, seqs, pool, refill=True)
    eng = DecodeEngine(w, arena_tokens=64 * 10, log_events=False)
    src = DeviceSources(w, eng, torch)
    eng.start(src.prefill)
    src.size_for(max(eng.n_active, 1))
    for _ in range(16):
        if eng.n_active == 0:
            break
        eng.step(src.tensors, src.prefill)
    torch.cuda.synchronize()
    eng.close()


def run_workload(name, args, torch, cpu_budget_s):
    from paper_2306_06000_amd import binding as s3
    from paper_2306_06000_amd.engine import DecodeEngine

    w = make_workload(name, args)
    shared_kv = w.kv_heads < w.n_heads  # not one of the paper's models: measured as a widening, not the headline
    steps = args.steps if args.steps is not None else DEFAULT_STEPS[name][0]
    warmup = args.warmup if args.warmup is not None else DEFAULT_STEPS[name][1]
    t_setup = time.perf_counter()
    eng = DecodeEngine(w, log_events=False, fused=not args.unfused, on_nomem=args.on_nomem)
    for pname, val in (("variant", args.variant if args.variant >= 0 else None), ("chunk", args.chunk or None),
                       ("grid_blocks", args.grid_blocks or None), ("classes", args.classes or None),
                       ("merge_sync", args.merge_sync or None), ("gqa_merge", args.gqa_merge if args.gqa_merge >= 0 else None),
                       ("gqa_stream", args.gqa_stream if args.gqa_stream >= 0 else None),
                       ("gqa_dynamic", args.gqa_dynamic if args.gqa_dynamic >= 0 else None)):
        if val is not None:
            s3.check(s3.s3_kv_set_param(eng.arena, pname, val), pname)
    src = DeviceSources(w, eng, torch)
    eng.start(src.prefill, stop_when_full=(name == "c3"))
    src.size_for(max(eng.n_active, 1))
    torch.cuda.synchronize()
    # working clocks, and what a plain streaming read reaches here: ~40 ms of back-to-back reads of (up to) 1 GB
    probe_bytes = min(eng.arena_mem.numel(), 1 << 30) & ~0xFFFF
    st, probe_gbps = s3.s3_kv_probe_bandwidth(eng.arena, probe_bytes, 0, max(4, int(0.04 * 5e12 / probe_bytes)))
    s3.check(st, "s3_kv_probe_bandwidth")
    setup_s = time.perf_counter() - t_setup
    flush = torch.empty(args.flush_mb << 20, dtype=torch.uint8, device=eng.dev) if args.flush_mb else None

    def timed_pass(evented, warm):
        """`warm` untimed steps, then `steps` timed decode steps; -> (bytes, sequence-steps, per-launch bytes, steps
        done, wall s, host enqueue s, lengths at the start of the timed steps)."""
        if evented:
            s3.check(s3.s3_kv_set_param(eng.arena, "profile", 1))
        total_bytes, seq_steps, launch_bytes, done = 0, 0, [], 0
        # The interpreter's cyclic garbage collector is kept out of the timed region (a full collection takes
        # tens of milliseconds here and would land on whichever step triggers it): collect now, resume after.
        gc.collect()
        gc.disable()
        # the collection above left the device idle for tens of milliseconds, long enough for its clocks to fall
        # back; a serving loop never pauses like that, so the device is kept streaming (the library's read probe,
        # about 10 ms) right up to the synchronisation that opens the timed region
        tail = torch.cuda.Event()
        tail.record()  # created and used once before the region: an event's first use costs tens of microseconds
        s3.check(s3.s3_kv_probe_bandwidth(eng.arena, probe_bytes, 0, max(2, int(0.01 * 5e12 / probe_bytes)))[0], "probe")
        # the warm-up steps come last, right before the synchronisation that opens the region: they leave the
        # interpreter's and the library's step path hot in the host's caches and the device at its working clocks
        for _ in range(warm):
            if eng.n_active:
                eng.step(src.tensors, src.prefill)
        if evented:  # warm-up launches are not part of the evented sample
            s3.check(s3.s3_kv_set_param(eng.arena, "profile", 1))
        lens0 = (eng.len.copy(), eng.n_grown, eng.n_retired)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            if eng.n_active == 0:  # drain runs: every sequence has finished
                break
            if flush is not None:
                flush.fill_(1)
            eng.step(src.tensors, src.prefill)
            done += 1
            total_bytes += eng.last_step_bytes
            seq_steps += eng.last_step_seqs
            launch_bytes.append(eng.last_step_bytes)
        t_enqueue = time.perf_counter() - t0  # host time to enqueue every step (no device wait in it)
        # the closing synchronisation is awaited by polling an event recorded behind the last step: a blocking wait
        # puts the host thread to sleep, and its wake-up (tens of microseconds) would be charged to a region that
        # at the driver's 20 steps of C1 lasts little more than a millisecond
        tail.record()
        while not tail.query():
            pass
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        gc.enable()
        return total_bytes, seq_steps, launch_bytes, done, dt, t_enqueue, lens0

    total_bytes, seq_steps, _lb, steps_done, dt, t_enqueue, (lens_at_start, grown0, retired0) = timed_pass(False, warmup)
    grown1, retired1 = eng.n_grown, eng.n_retired
    res = {
        "workload": w.name, "value": round(total_bytes / dt / 1e9, 2), "unit": "GB/s",
        "pct_of_peak_hbm": round(100 * total_bytes / dt / 1e9 / PEAK_HBM_GBPS, 2),
        "steps": steps_done, "warmup": warmup, "ms_per_step": round(dt / max(steps_done, 1) * 1e3, 5),
        "seq_steps_per_s": round(seq_steps / dt, 1),
        "host_enqueue_ms_per_step": round(t_enqueue / max(steps_done, 1) * 1e3, 5),
        "dtype": {0: "f16", 1: "bf16", 3: "e4m3 rows, 16-bit queries, f32 arithmetic"}[w.dtype],
        "plain_read_probe_GBps": round(probe_gbps, 1), "setup_s": round(setup_s, 2),
        "config": {"workload": w.name, "batch": int(lens_at_start.size), "n_layers": w.n_layers,
                   "n_heads": w.n_heads, "n_kv_heads": w.kv_heads, "head_dim": w.head_dim,
                   "mean_context_at_start": round(float(lens_at_start.mean()), 1) if lens_at_start.size else 0.0,
                   "batch_at_end": int(eng.n_active), "refill": bool(w.refill),
                   "grows": grown1 - grown0, "retired": retired1 - retired0,
                   "swapped_out": eng.n_swapped_out, "swapped_in": eng.n_swapped_in, "compactions": eng.n_compactions,
                   "dropped": eng.n_evicted, "on_nomem": args.on_nomem,
                   "arena_GB": round(eng.arena_mem.numel() / 1e9, 3),
                   "algorithmic_GB_per_step": round(total_bytes / max(steps_done, 1) / 1e9, 4),
                   "algorithmic_bytes_per_launch": int(total_bytes / max(steps_done * w.n_layers, 1)),
                   "path": "quantising append + shared-kv matrix-core attention over 8-bit rows + merge per layer" if shared_kv and w.dtype == 3 else
                           "shared-kv attention kernel (+ append launch for the vector-ALU kernel) + merge per layer" if shared_kv else
                           "one s3_decode_step kernel per layer (quantises and appends the new row, attends over 8-bit rows, merges)" if w.dtype == 3 else
                           "append+attention+merge kernels" if args.unfused else "one s3_decode_step kernel per layer",
                   "variant": s3.s3_kv_get_param(eng.arena, "variant")[1],
                   "chunk": s3.s3_kv_get_param(eng.arena, "chunk")[1]},
    }
    if not args.no_kernel_events and eng.n_active > 0:
        ev_bytes, _ss, step_bytes, ev_steps, ev_dt, _te, _l0 = timed_pass(True, 0)
        launches = s3.s3_kv_get_param(eng.arena, "profile_launches")[1]
        part_ns = s3.s3_kv_get_param(eng.arena, "profile_partial_ns")[1]
        merge_ns = s3.s3_kv_get_param(eng.arena, "profile_merge_ns")[1]
        assert launches == ev_steps * w.n_layers, (launches, ev_steps, w.n_layers)
        per_launch_bytes = ev_bytes / max(launches, 1)
        avg_us = part_ns / max(launches, 1) / 1e3
        achieved = per_launch_bytes / (avg_us * 1e-6) / 1e9 if avg_us > 0 else 0.0
        kind = s3.s3_kv_get_param(eng.arena, "kernel_kind")[1]
        kernel = {1: "attn_gqa_kernel", 2: "attn_gqa_mfma_kernel", 3: "attn_fp8_kernel", 4: "attn_gqa_mfma_kernel"}.get(
            kind, "attn_partial_kernel" if args.unfused else "attn_step_kernel")
        traffic, traffic_ref = read_traffic(kernel, name)
        res["roofline"] = {"bound": "hbm", "kernel": kernel, "achieved": round(achieved, 1),
                           "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBPS, 4),
                           "traffic": traffic, "traffic_ref_algorithmic": traffic_ref,
                           "traffic_over_algorithmic": round(traffic / traffic_ref, 4) if traffic and traffic_ref else None,
                           "avg_kernel_us": round(avg_us, 2),
                           "kernel_us_p10_p50_p90": [round(s3.s3_kv_get_param(eng.arena, f"profile_p{q}_ns")[1] / 1e3, 2)
                                                     for q in (10, 50, 90)],
                           "timed_launches": launches, "algorithmic_bytes_per_launch": int(per_launch_bytes),
                           "pass": f"pass 2: the {ev_steps} steps after the timed region, every attention launch bracketed",
                           "pass2_whole_region_GBps": round(ev_bytes / ev_dt / 1e9, 1)}
        if args.unfused:
            res["roofline"]["avg_merge_kernel_us"] = round(merge_ns / max(launches, 1) / 1e3, 2)
        s3.check(s3.s3_kv_set_param(eng.arena, "profile", 0))
    if args.flush_mb:
        res["config"]["cache_flush_MB_between_steps"] = args.flush_mb
    if cpu_budget_s > 0:
        res["cpu_baseline"] = cpu_baseline(w, lens_at_start, cpu_budget_s)
    eng.close()
    del eng, src, flush
    gc.collect()
    torch.cuda.empty_cache()
    return res


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2306_06000_amd import binding as s3

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    s3.lib()
    prime_code_paths(torch)
    names = TARGETS if args.workload == "all" else (args.workload,)
    results, errors = [], {}
    for i, name in enumerate(names):
        budget = 0.0 if args.no_cpu_baseline else (12.0 if i == 0 else 3.0)
        try:
            results.append(run_workload(name, args, torch, budget))
        except Exception as e:  # one workload that cannot run (e.g. no 200 GB free) must not hide the others
            if len(names) == 1:
                raise
            errors[name] = f"{type(e).__name__}: {e}"
            gc.collect()
            torch.cuda.empty_cache()
    assert results, errors
    head = results[0]
    line = {"metric": METRIC, "value": head["value"], "unit": "GB/s", "n_gpus": 1, "steps": head["steps"],
            "warmup": head["warmup"], "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": head["dtype"], "data": "synthetic",
            "pct_of_peak_hbm": head["pct_of_peak_hbm"], "seq_steps_per_s": head["seq_steps_per_s"],
            "host_enqueue_ms_per_step": head["host_enqueue_ms_per_step"], "config": head["config"]}
    for key in ("roofline", "cpu_baseline", "plain_read_probe_GBps"):
        if key in head:
            line[key] = head[key]
    if len(results) > 1 or errors:
        line["per_config"] = [{k: r[k] for k in ("workload", "value", "unit", "pct_of_peak_hbm", "steps", "warmup", "ms_per_step",
                                                  "seq_steps_per_s", "host_enqueue_ms_per_step", "dtype",
                                                  "plain_read_probe_GBps", "roofline", "cpu_baseline", "config") if k in r}
                              for r in results]
        if errors:
            line["errors"] = errors
    print(json.dumps(line))


if __name__ == "__main__":
    main()
