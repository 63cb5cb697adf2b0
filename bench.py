#!/usr/bin/env python3
"""Benchmark of the GPU LSM key index on one MI355X.

A step is one pass of the whole index hot path over one batch of synthetic input:
  1. lsm_compact      tiered 16-way merge of 16 runs x 4,194,304 entries (4 GiB) into the last level
  2. read back n_out  (the host needs it to install the new run)
  3. lsm_build_fences fence index (stride 64) of the merged run
  4. lsm_probe        one batch of 4,096 longest-prefix requests against the merged run
Inputs are generated on the GPU before the timed region and stay resident in HBM.

Prints one JSON line; see the design doc for the definition of every field.
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

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E


def cpu_baseline(runs_gpu, sample_per_run: int):
    """The CPU checker (single thread, as it stands) on a bounded sample of the same workload:
    the first `sample_per_run` entries of every run."""
    from oracle import lsm_oracle
    lsm_oracle.build()
    sample = [lsm_oracle.as_run(r[:sample_per_run].cpu()) for r in runs_gpu]
    n_in = sum(r.shape[0] for r in sample)
    t0 = time.perf_counter()
    out = lsm_oracle.compact(sample, lsm_oracle.FLAG_BOTTOMMOST)
    dt = time.perf_counter() - t0
    return {"value": n_in / dt, "unit": "merged entries/s", "cores": 1, "kind": "oracle",
            "sample": f"heap merge of the first {sample_per_run} entries of each of the {len(sample)} runs "
                      f"({n_in} in, {out.shape[0]} out, {dt:.1f} s)"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scale", type=int, default=1, help="divide the workload size (1 = the full configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the index shards by key range without any exchange, "
              "see DESIGN.md); run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2511_16138_amd as g
    from workloads import lsm

    if not os.path.exists(g.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    t0 = time.perf_counter()
    w = lsm.config3(device=dev, scale=args.scale)
    runs = [r.contiguous() for r in w.runs]
    n_in = sum(int(r.shape[0]) for r in runs)
    q, nb = lsm.queries_config4(w, 4096)
    n_keys = int(nb.sum().item())
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t0

    out = torch.empty((n_in, 8), dtype=torch.int64, device=dev)
    n_out_d = torch.zeros(1, dtype=torch.int64, device=dev)
    ws = torch.empty(g.lsm_compact_workspace_bytes([int(r.shape[0]) for r in runs]), dtype=torch.uint8, device=dev)
    fences = torch.empty(((n_in + 63) // 64, 4), dtype=torch.int64, device=dev)
    hit_len = torch.empty(q.shape[0], dtype=torch.int32, device=dev)
    hits = torch.empty((q.shape[0], q.shape[1], 2), dtype=torch.int64, device=dev)
    del w.universe.keys  # free what the steps do not need
    torch.cuda.empty_cache()

    stream = torch.cuda.current_stream()

    def mk_events(n):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n)]
        for e in evs:
            e.record(stream)  # creates the underlying hipEvent_t; the library re-records it
        return evs

    n_total = args.warmup + args.steps
    ev_part, ev_merge0, ev_merge1 = mk_events(n_total), mk_events(n_total), mk_events(n_total)
    ev_c1, ev_f1, ev_p1 = mk_events(n_total), mk_events(n_total), mk_events(n_total)
    torch.cuda.synchronize()

    def step(i):
        g.lsm_compact(runs, g.LSM_BOTTOMMOST, out=out, n_out=n_out_d, workspace=ws,
                      events=(ev_part[i].cuda_event, ev_merge0[i].cuda_event, ev_merge1[i].cuda_event))
        n_out = int(n_out_d.item())  # device -> host, synchronises
        ev_c1[i].record(stream)
        merged = out[:n_out]
        f = fences[: (n_out + 63) // 64]
        g.lsm_build_fences(merged, 64, out=f)
        ev_f1[i].record(stream)
        g.lsm_probe(q, nb, [g.TreeRun(merged, f, 64, 1)], hit_len=hit_len, hits=hits)
        ev_p1[i].record(stream)
        return n_out

    for i in range(args.warmup):
        n_out = step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.warmup, n_total):
        n_out = step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    sl = range(args.warmup, n_total)
    mean = lambda xs: sum(xs) / max(1, len(xs))
    ms_partition = mean([ev_part[i].elapsed_time(ev_merge0[i]) for i in sl])
    ms_merge = mean([ev_merge0[i].elapsed_time(ev_merge1[i]) for i in sl])
    ms_compact = mean([ev_part[i].elapsed_time(ev_merge1[i]) for i in sl])
    ms_fence = mean([ev_c1[i].elapsed_time(ev_f1[i]) for i in sl])
    ms_probe = mean([ev_f1[i].elapsed_time(ev_p1[i]) for i in sl])
    ms_step = elapsed * 1e3 / args.steps

    algo_bytes = 64 * (n_in + n_out)  # every input entry read once, every survivor written once
    achieved = algo_bytes / (ms_merge * 1e-3) / 1e9
    result = {
        "metric": "compaction merged entries/s (HBM GB/s % peak); prefix probes/s",
        "value": n_in / (ms_step * 1e-3),
        "unit": "merged entries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u64", "data": "synthetic",
        "config": {"workload": ("configs[2]: tiered 16-way merge of 16 runs x %d entries into the last level "
                                "(20%% duplicated keys, 5%% tombstones), then fence build and one batch of 4096 "
                                "longest-prefix requests against the merged run") % (n_in // 16),
                   "n_in": n_in, "n_out": n_out, "probe_requests": int(q.shape[0]), "probe_keys": n_keys,
                   "scale_divisor": args.scale},
        "compact_entries_per_s": n_in / (ms_compact * 1e-3),
        "compact_hbm_gbps": algo_bytes / (ms_compact * 1e-3) / 1e9,
        "compact_hbm_frac_of_peak": algo_bytes / (ms_compact * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "probes_per_s": int(q.shape[0]) / (ms_probe * 1e-3),
        "probe_key_lookups_per_s": n_keys / (ms_probe * 1e-3),
        "ms": {"partition_kernels": ms_partition, "merge_kernel": ms_merge, "compact_total": ms_compact,
               "fence_build": ms_fence, "probe_batch": ms_probe, "generate_inputs_s": gen_s},
        "roofline": {"bound": "hbm", "kernel": "merge_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": None, "algorithmic_bytes": algo_bytes},
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(runs, max(1, (1 << 21) // args.scale))
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
