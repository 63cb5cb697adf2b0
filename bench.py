#!/usr/bin/env python3
"""Benchmark of the GPU LSM key index on one MI355X.

A step is one pass of the whole index hot path over one batch of synthetic input:
  1. lsm_compact      tiered 16-way merge of 16 runs x 4,194,304 entries (4 GiB) into the last level
  2. read back n_out  (the host needs it to install the new run)
  3. lsm_build_fences fence index (stride 64) of the merged run
  4. lsm_probe        one batch of 4,096 longest-prefix requests against the merged run
Inputs are generated on the GPU before the timed region and stay resident in HBM.

Prints one JSON line.  `value` = input entries of the compaction per second of whole step; `roofline` = the merge
kernel's algorithmic bytes (64 per input entry + 64 per survivor) over its duration against the HBM peak, `traffic`
its measured HBM bytes; `cpu_baseline` = the CPU checker on a bounded sample; the other sections are labelled.
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
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "compaction_cfg3_tiered16_hbm_traffic.md")
MERGE_KERNEL_SOURCE = os.path.join(ROOT, "paper_2511_16138_amd", "csrc", "lsm_compact.hip")


def measured_traffic(section: str, source: str):
    """HBM bytes per launch of a kernel from the rocprofv3 FETCH_SIZE / WRITE_SIZE summary under profiles/ (the
    line `traffic <section>: bytes_per_launch=... source_sha256=...`).  None when there is no such line or when the
    kernel's source file has changed since the counters were taken."""
    import hashlib
    import re
    try:
        text = open(TRAFFIC_PROFILE).read()
        sha = hashlib.sha256(open(source, "rb").read()).hexdigest()
    except OSError:
        return None
    m = re.search(r"traffic %s: bytes_per_launch=(\d+) source_sha256=([0-9a-f]{64})" % re.escape(section), text)
    return int(m.group(1)) if m and m.group(2) == sha else None


def host_description():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"cpu_model": model, "logical_cpus": os.cpu_count()}


def cpu_baseline(sample_runs, threads: int):
    """The CPU checker as it stands on the same workload (host copies made by the caller): (i) the single-thread heap
    merge, (ii) the same merge over `threads` key ranges at once - splitters are every (n / threads)-th key of the
    largest run, every thread merges the slices of all runs inside its range, the outputs are concatenated."""
    import bisect
    from concurrent.futures import ThreadPoolExecutor

    from oracle import lsm_oracle
    lsm_oracle.build()
    sample = [lsm_oracle.as_run(r) for r in sample_runs]
    sample_per_run = sample[0].shape[0]
    n_in = sum(r.shape[0] for r in sample)
    t0 = time.perf_counter()
    out = lsm_oracle.compact(sample, lsm_oracle.FLAG_BOTTOMMOST)
    dt = time.perf_counter() - t0
    host = host_description()
    result = {"value": n_in / dt, "unit": "merged entries/s", "cores": 1, "kind": "oracle",
              "sample": f"heap merge of all {sample_per_run} entries of each of the {len(sample)} runs "
                        f"({n_in} in, {out.shape[0]} out, {dt:.1f} s)", "host": host}

    class KeysOf:  # run[i].key as bytes, for bisect (order = the checker's key order = bytes order)
        def __init__(self, run):
            self.run = run

        def __len__(self):
            return self.run.shape[0]

        def __getitem__(self, i):
            return self.run[i, :32].tobytes()

    t0 = time.perf_counter()
    largest = max(sample, key=lambda r: r.shape[0])
    splitters = [largest[(i * largest.shape[0]) // threads, :32].tobytes() for i in range(1, threads)]
    cuts = [[0] + [bisect.bisect_left(KeysOf(r), k) for k in splitters] + [r.shape[0]] for r in sample]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(lambda i: lsm_oracle.compact([r[c[i]:c[i + 1]] for r, c in zip(sample, cuts)],
                                                         lsm_oracle.FLAG_BOTTOMMOST), range(threads)))
    n_par = sum(p.shape[0] for p in parts)
    dt_par = time.perf_counter() - t0
    assert n_par == out.shape[0], "the range-partitioned merge gave another count"
    result["all_cores"] = {"value": n_in / dt_par, "unit": "merged entries/s", "cores": threads, "kind": "oracle",
                           "sample": f"the same merge over {threads} key ranges at once ({dt_par:.1f} s)"}
    return result


def probe_useful_bytes(nb, hit_len, hits, n_runs: int, filtered: bool, stride: int = 64):
    """Bytes a probe batch must move by the per-key formula: a request needs its hit_len found keys and the first
    missing one looked up; a lookup reads the 32-byte key, writes 16 bytes of result and, in every run it has to search
    until the key is resolved, the final 64-byte entry plus log2(stride) more entries of the in-page search (the fence
    levels above the page count as cached).  Without filters a found key searches run_idx + 1 runs and a missing one
    all runs; with filters only the run that holds the key, plus one 16-byte filter block per run consulted."""
    import math
    n = nb.to(hit_len.dtype)
    first_miss = (hit_len < n).sum().item()
    found = int(hit_len.sum().item())
    keys = found + int(first_miss)
    run_idx = (hits[..., 1] >> 32)  # high half of the second word
    col = __import__("torch").arange(hits.shape[1], device=hits.device)[None, :]
    searched_for_found = int(((run_idx + 1) * (col < hit_len[:, None])).sum().item())
    per_search = (1 + int(math.ceil(math.log2(stride)))) * 64
    if filtered:
        return keys * 48 + found * per_search + (searched_for_found + int(first_miss) * n_runs) * 16
    return keys * 48 + (searched_for_found + int(first_miss) * n_runs) * per_search


def filter_pipeline(g, torch, dev, runs, out, n_out_d, ws, fences, n_out: int):
    """What a compaction costs when the new run also gets its fence index and its Bloom filter (16 bits per key): the
    merge writes the fence keys and the keys' filter hashes in its own pass and the filter is built from the hashes;
    beside it the two separate builds from the finished run (from hashes computed by a pass over the run; by atomic
    operations on the filter).  Medians of five runs each."""
    import statistics
    n_in = int(out.shape[0])
    hashes = torch.empty(n_in, dtype=torch.int64, device=dev)
    n_blocks = g.lsm_bloom_blocks(n_out, 16)
    bws = torch.empty(max(g.lsm_bloom_workspace_bytes(n_out, n_blocks), 256), dtype=torch.uint8, device=dev)
    f_hashed = torch.empty((n_blocks, 4), dtype=torch.int32, device=dev)
    f_atomic = torch.empty((n_blocks, 4), dtype=torch.int32, device=dev)
    h2 = torch.empty(n_out, dtype=torch.int64, device=dev)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return statistics.median(ts)

    ms_compact = timed(lambda: g.lsm_compact(runs, g.LSM_BOTTOMMOST, out=out, n_out=n_out_d, workspace=ws, fences=fences, fence_stride=64,
                                             key_hashes=hashes))
    assert int(n_out_d.item()) == n_out
    ms_hashed = timed(lambda: g.lsm_build_bloom_hashed(hashes[:n_out], n_blocks, out=f_hashed, workspace=bws))
    index = torch.empty((g.lsm_hash_index_buckets(n_out), 8), dtype=torch.int64, device=dev)
    iws = torch.empty(max(g.lsm_hash_index_workspace_bytes(n_out), 256), dtype=torch.uint8, device=dev)
    ms_index = timed(lambda: g.lsm_build_hash_index(hashes[:n_out], out=index, workspace=iws))
    del index, iws
    ms_hash_keys = timed(lambda: g.lsm_hash_keys(out[:n_out], out=h2))
    ms_atomic = timed(lambda: g.lsm_build_bloom(out[:n_out], 16, out=f_atomic))
    assert torch.equal(f_hashed, f_atomic) and torch.equal(h2, hashes[:n_out]), "the two filter builds disagree"
    return {"workload": "the same compaction, new run with fence index and Bloom filter (16 bits per key, %d blocks)" % n_blocks,
            "compact_writing_fences_and_key_hashes_ms": ms_compact, "filter_from_hashes_ms": ms_hashed,
            "total_ms": ms_compact + ms_hashed, "merged_entries_per_s": n_in / ((ms_compact + ms_hashed) * 1e-3),
            "hash_index_from_hashes_ms": ms_index,
            "separate_builds": {"hash_keys_pass_over_the_run_ms": ms_hash_keys, "filter_by_atomics_ms": ms_atomic}}


def probe_config4(g, lsm, torch, dev, n_batches: int, scale: int):
    """Lookup-heavy configuration: batches of 4,096 longest-prefix requests (Zipf(0.99) prefixes, 30 % misses,
    up to 256 block keys each) against the 5-level, 100M-entry tree.  Returns probes/s and key lookups/s (medians over
    the batches) and the rate of useful bytes against the HBM peak."""
    import statistics
    w = lsm.config4(device=dev, scale=scale)
    plain = [g.TreeRun(r, g.lsm_build_fences(r, 64), 64, i + 1) for i, r in enumerate(w.runs)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    filtered = []
    for t in plain:   # long runs: from the keys' hashes; short ones: one workgroup
        n = int(t.run.shape[0])
        n_blocks = g.lsm_bloom_blocks(n, 16)
        bloom = (g.lsm_build_bloom_hashed(g.lsm_hash_keys(t.run), n_blocks) if n >= (1 << 20) and g.lsm_bloom_workspace_bytes(n, n_blocks)
                 else g.lsm_build_bloom(t.run, 16))
        filtered.append(g.TreeRun(t.run, t.fences, 64, t.level, bloom))
    torch.cuda.synchronize()
    bloom_build_ms = (time.perf_counter() - t0) * 1e3
    batches = [lsm.queries_config4(w, 4096, stream=b) for b in range(n_batches)]
    hit_len = torch.empty(4096, dtype=torch.int32, device=dev)
    hits = torch.empty((4096, 256, 2), dtype=torch.int64, device=dev)

    def timed(call):
        for q, nb in batches[:2]:
            call(q, nb)
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in batches]
        for (q, nb), (e0, e1) in zip(batches, evs):
            e0.record()
            call(q, nb)
            e1.record()
        torch.cuda.synchronize()
        return statistics.median(e0.elapsed_time(e1) for e0, e1 in evs)

    ms_plain = timed(lambda q, nb: g.lsm_probe(q, nb, plain, hit_len=hit_len, hits=hits))
    plain_len = hit_len.clone()
    useful_plain = probe_useful_bytes(batches[-1][1], hit_len, hits, len(plain), False)
    ms = timed(lambda q, nb: g.lsm_probe(q, nb, filtered, hit_len=hit_len, hits=hits))
    assert bool((plain_len == hit_len).all()), "filters changed a probe result"
    useful = probe_useful_bytes(batches[-1][1], hit_len, hits, len(filtered), True)
    # length of the prefix only, by search over the length (the generator's data is prefix-closed)
    ms_len = timed(lambda q, nb: g.lsm_probe_length(q, nb, filtered, hit_len=hit_len))
    assert bool((plain_len == hit_len).all()), "the search over the prefix length gave another length"
    ms_len_plain = timed(lambda q, nb: g.lsm_probe_length(q, nb, plain, hit_len=hit_len))
    # hash indices on every run (one 64-byte read finds or rules out a key): with the filters, and in their place
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    indices = [g.lsm_build_hash_index(g.lsm_hash_keys(t.run)) for t in plain]
    torch.cuda.synchronize()
    index_build_ms = (time.perf_counter() - t0) * 1e3
    both = [g.TreeRun(t.run, t.fences, 64, t.level, t.bloom, ix) for t, ix in zip(filtered, indices)]
    ms_ix = timed(lambda q, nb: g.lsm_probe(q, nb, both, hit_len=hit_len, hits=hits))
    assert bool((plain_len == hit_len).all()), "hash indices changed a probe result"
    only_ix = [g.TreeRun(t.run, t.fences, 64, t.level, None, ix) for t, ix in zip(plain, indices)]
    ms_ix_plain = timed(lambda q, nb: g.lsm_probe(q, nb, only_ix, hit_len=hit_len, hits=hits))
    assert bool((plain_len == hit_len).all()), "hash indices changed a probe result"
    ms_ix_len = timed(lambda q, nb: g.lsm_probe_length(q, nb, both, hit_len=hit_len))
    assert bool((plain_len == hit_len).all()), "hash indices changed a prefix length"
    keys = sum(int(nb.sum().item()) for _, nb in batches) / n_batches
    traffic = measured_traffic("probe_kernel_cfg4_filtered", os.path.join(ROOT, "paper_2511_16138_amd", "csrc", "lsm_probe.hip"))
    return {"workload": "configs[3]: 5-level tree of %d entries, batches of 4096 requests, Bloom filters of 16 bits per key on every run"
                        % sum(int(r.shape[0]) for r in w.runs),
            "batches_timed": n_batches, "ms_per_batch": ms, "probes_per_s": 4096 / (ms * 1e-3),
            "requested_keys_per_s": keys / (ms * 1e-3), "mean_hit_len_last_batch": float(plain_len.float().mean().item()),
            "probe_roofline": {"bound": "hbm", "kernel": "probe_kernel", "achieved": useful / (ms * 1e-3) / 1e9,
                               "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": useful / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                               "useful_bytes_per_batch": useful, "traffic": traffic},
            "without_filters": {"ms_per_batch": ms_plain, "probes_per_s": 4096 / (ms_plain * 1e-3),
                                "useful_bytes_per_batch": useful_plain,
                                "useful_gbps": useful_plain / (ms_plain * 1e-3) / 1e9},
            "length_only": {"ms_per_batch": ms_len, "probes_per_s": 4096 / (ms_len * 1e-3),
                            "without_filters_ms_per_batch": ms_len_plain},
            "with_hash_indices": {"ms_per_batch": ms_ix, "probes_per_s": 4096 / (ms_ix * 1e-3),
                                  "requested_keys_per_s": keys / (ms_ix * 1e-3),
                                  "without_filters_ms_per_batch": ms_ix_plain, "length_only_ms_per_batch": ms_ix_len,
                                  "index_bytes": sum(int(ix.numel()) * 8 for ix in indices), "build_ms_all_runs": index_build_ms,
                                  "traffic": measured_traffic("probe_kernel_cfg4_filtered_indexed",
                                                              os.path.join(ROOT, "paper_2511_16138_amd", "csrc", "lsm_probe.hip"))},
            "bloom_build_ms_all_runs": bloom_build_ms}


def mixed_config5(g, lsm, torch, dev, scale: int):
    """Mixed shifting workload on the 6-level, 400M-entry tree: flushes, compactions chosen by the
    adaptive controller and probe batches, replayed twice: by the library's own driver (lsm_driver_*) and by the Python
    driver over the single entry points.  Probe batches are generated before the clock starts."""
    from paper_2511_16138_amd.tree import AdaptiveLsmTree, GpuBackend
    tr = lsm.config5(device=dev, tree_total=400_000_000 // scale, buffer_entries=max(36, 3600 // scale),
                     ops_per_phase=(1 << 18) // scale)
    batches = {i: tr.probe_batch(i) for kind, i, _ in tr.events if kind == "probe"}

    def replay(tree):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        t_probe = 0.0
        for (kind, i, _phase), n_writes in zip(tr.events, tr.write_ops_between):
            if n_writes:
                tree.note_writes(n_writes)
            if kind == "flush":
                tree.flush(tr.flush_runs[i])
            else:
                torch.cuda.synchronize()
                tp = time.perf_counter()
                tree.probe(*batches[i])
                torch.cuda.synchronize()
                t_probe += time.perf_counter() - tp
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        trace = list(tree.trace)
        comp = [e for e in trace if e[0] == "compact"]
        merged = sum(e[3] for e in comp)
        n_probe = sum(e[1] for e in trace if e[0] == "probe")
        return trace, {"seconds": dt, "compactions": len(comp), "entries_merged": merged,
                       "merged_entries_per_s_incl_host": merged / max(dt - t_probe, 1e-9),
                       "probes": n_probe, "probes_per_s_incl_host": n_probe / max(t_probe, 1e-9)}

    window = 16 * tr.batch_requests
    native = g.LsmDriver(tr.buffer_entries, size_ratio=tr.size_ratio, window_ops=window, t_grid=(2, 16), bloom_bits=16)
    for level, r in enumerate(tr.workload.runs):
        native.load_run(level + 1, r)
    native_trace, native_res = replay(native)
    native_sizes, at = [], 0
    runs = native.tree()
    for _t, _k, n_runs in native.levels():
        native_sizes.append([int(t.run.n) for t in runs[at:at + n_runs]])
        at += n_runs
    native.close()
    tree = AdaptiveLsmTree(GpuBackend(bloom_bits=16), tr.buffer_entries, size_ratio=tr.size_ratio, window_ops=window, t_grid=(2, 16))
    for level, r in enumerate(tr.workload.runs):
        tree.load_level(level, [r])
    trace, res = replay(tree)
    sizes = [[r.n for r in lv] for lv in tree.levels]
    assert trace == native_trace and sizes == native_sizes, "the two drivers built different trees"
    return {"workload": "configs[4]: %d-level tree of %d entries, %d flushes of %d entries, %d probe batches"
                        % (len(tr.workload.runs), sum(int(r.shape[0]) for r in tr.workload.runs), tr.flush_runs.shape[0],
                           tr.buffer_entries, len(batches)),
            **native_res, "driver": "lsm_driver_* (C++, in the library)",
            "python_driver": res,
            "policy_trace_T_K": [e[1:3] for e in trace if e[0] == "policy"],
            "final_level_sizes": sizes}


def sharded_config5(g, lsm, torch, dev, n_shards: int, scale: int):
    """Batched small compactions: `n_shards` independent trees (key-range shards of one index, or tenants), each with
    the mixed workload at 1 / n_shards of its size, written to in step.  The same flush rounds are replayed twice: every
    tree's compactions on their own (one lsm_compact per compaction), and the compactions of a round in one
    lsm_compact_batch.  Probe batches are left out of this section (they are the same calls either way)."""
    from paper_2511_16138_amd.tree import AdaptiveLsmTree, GpuBackend, ShardedLsmTrees
    from workloads import rng
    traces = [lsm.config5(device=dev, seed=rng.SEED + 1000 * i, tree_total=400_000_000 // scale // n_shards,
                          buffer_entries=max(36, 3600 // scale), ops_per_phase=(1 << 18) // scale // n_shards) for i in range(n_shards)]
    rounds = max(int(tr.flush_runs.shape[0]) for tr in traces)

    def build():
        backend = GpuBackend(bloom_bits=16)
        trees = [AdaptiveLsmTree(backend, tr.buffer_entries, size_ratio=tr.size_ratio, window_ops=16 * tr.batch_requests,
                                 t_grid=(2, 16)) for tr in traces]
        for tr, tree in zip(traces, trees):
            for level, r in enumerate(tr.workload.runs):
                tree.load_level(level, [r])
        return backend, trees

    def replay(batched: bool):
        backend, trees = build()
        sharded = ShardedLsmTrees(trees, backend)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for f in range(rounds):
            runs = [tr.flush_runs[f] if f < tr.flush_runs.shape[0] else None for tr in traces]
            if batched:
                sharded.flush_all(runs)
            else:
                for tree, run in zip(trees, runs):
                    if run is not None:
                        tree.flush(run)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        comp = [e for t in trees for e in t.trace if e[0] == "compact"]
        return dt, len(comp), sum(e[3] for e in comp), [[r.n for r in lv] for lv in trees[0].levels]

    def replay_library(batched: bool):
        """The same rounds through the library's own driver: lsm_driver_flush per tree, or lsm_driver_flush_many per round."""
        trees = [g.LsmDriver(tr.buffer_entries, size_ratio=tr.size_ratio, window_ops=16 * tr.batch_requests, t_grid=(2, 16),
                             bloom_bits=16) for tr in traces]
        for tr, tree in zip(traces, trees):
            for level, r in enumerate(tr.workload.runs):
                tree.load_run(level + 1, r)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for f in range(rounds):
            runs = [tr.flush_runs[f] if f < tr.flush_runs.shape[0] else None for tr in traces]
            if batched:
                g.lsm_driver_flush_many(trees, runs)
            else:
                for tree, run in zip(trees, runs):
                    if run is not None:
                        tree.flush(run)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        comp = [e for t in trees for e in t.trace if e[0] == "compact"]
        first = trees[0].tree()
        shape, at = [], 0
        for _t, _k, n_runs in trees[0].levels():
            shape.append([int(t.run.n) for t in first[at:at + n_runs]])
            at += n_runs
        for t in trees:
            t.close()
        return dt, len(comp), sum(e[3] for e in comp), shape

    dt_one, n_comp, merged, shape_one = replay(False)
    dt_batch, n_comp_b, merged_b, shape_batch = replay(True)
    assert (n_comp, merged, shape_one) == (n_comp_b, merged_b, shape_batch), "the batched replay built another tree"
    lib_one, lib_batch = replay_library(False), replay_library(True)
    assert lib_one[1:] == (n_comp, merged, shape_one) and lib_batch[1:] == (n_comp, merged, shape_one), "the library's driver built another tree"
    return {"workload": "%d independent trees of %d entries, %d flush rounds of %d entries per tree"
                        % (n_shards, sum(int(r.shape[0]) for r in traces[0].workload.runs), rounds, traces[0].buffer_entries),
            "compactions": n_comp, "entries_merged": merged,
            "one_call_per_compaction": {"seconds": dt_one, "merged_entries_per_s_incl_host": merged / dt_one},
            "batched": {"seconds": dt_batch, "merged_entries_per_s_incl_host": merged / dt_batch},
            "speedup": dt_one / dt_batch,
            "library_driver": {"one_call_per_compaction": {"seconds": lib_one[0], "merged_entries_per_s_incl_host": merged / lib_one[0]},
                               "batched": {"seconds": lib_batch[0], "merged_entries_per_s_incl_host": merged / lib_batch[0]}}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scale", type=int, default=1, help="divide the workload size (1 = the full configuration)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe-config", action="store_true", help="skip the extra probe measurement on the 100M-entry tree")
    ap.add_argument("--no-mixed", action="store_true", help="skip the replay of the mixed workload on the 400M-entry tree")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="before the steps, run a plain streaming kernel (dst = src + 1 over 1 GiB of int64, 5 launches) "
                         "whose HBM bytes are known; it scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU only (the index shards by key range without any exchange); "
              "run with --gpus 1", file=sys.stderr)
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

    if args.calibrate_copy:
        src = torch.arange(1 << 27, dtype=torch.int64, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.add(src, 1, out=dst)  # reads 2^30 bytes, writes 2^30 bytes per launch
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

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
        if not 0 <= n_out <= n_in:
            raise RuntimeError(f"lsm_compact reported a device-side failure (n_out = {n_out})")
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

    import statistics
    sl = range(args.warmup, n_total)
    mean = lambda xs: sum(xs) / max(1, len(xs))
    med = lambda xs: statistics.median(xs) if xs else 0.0
    t_part = [ev_part[i].elapsed_time(ev_merge0[i]) for i in sl]
    t_merge = [ev_merge0[i].elapsed_time(ev_merge1[i]) for i in sl]
    t_compact = [ev_part[i].elapsed_time(ev_merge1[i]) for i in sl]
    t_fence = [ev_c1[i].elapsed_time(ev_f1[i]) for i in sl]
    t_probe = [ev_f1[i].elapsed_time(ev_p1[i]) for i in sl]
    ms_partition, ms_merge, ms_compact, ms_fence, ms_probe = med(t_part), med(t_merge), med(t_compact), med(t_fence), med(t_probe)
    ms_merge_mean = mean(t_merge)  # the roofline figure divides by the average launch duration
    ms_step = elapsed * 1e3 / args.steps

    algo_bytes = 64 * (n_in + n_out)  # every input entry read once, every survivor written once
    achieved = algo_bytes / (ms_merge_mean * 1e-3) / 1e9
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
               "fence_build": ms_fence, "probe_batch": ms_probe, "statistic": "median over the timed steps",
               "merge_kernel_mean": ms_merge_mean, "generate_inputs_s": gen_s},
        "roofline": {"bound": "hbm", "kernel": "merge_kernel", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic("merge_kernel_cfg3", MERGE_KERNEL_SOURCE) if args.scale == 1 else None,
                     "algorithmic_bytes": algo_bytes},
    }
    # second denominator: a plain device-to-device copy that moves the same number of bytes (half read, half written)
    half = algo_bytes // 2 // 8
    src = torch.empty(half, dtype=torch.int64, device=dev).random_()
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbps = 2 * half * 8 / (c0.elapsed_time(c1) / 5 * 1e-3) / 1e9
    result["copy_ceiling_gbps"] = copy_gbps
    result["compact_frac_of_copy_ceiling"] = result["compact_hbm_gbps"] / copy_gbps
    result["merge_kernel_frac_of_copy_ceiling"] = achieved / copy_gbps
    del src, dst
    result["filter_pipeline"] = filter_pipeline(g, torch, dev, runs, out, n_out_d, ws, fences, n_out)
    cpu_sample = None if args.no_cpu_baseline else [r.cpu() for r in runs]  # the whole workload: a few seconds for the checker
    del runs, out, fences, q, hits, w
    torch.cuda.empty_cache()
    if not args.no_probe_config:
        result["probe_config"] = probe_config4(g, lsm, torch, dev, 16, args.scale)
        torch.cuda.empty_cache()
    if not args.no_mixed:
        result["mixed_config"] = mixed_config5(g, lsm, torch, dev, args.scale)
        torch.cuda.empty_cache()
        result["sharded_mixed_config"] = sharded_config5(g, lsm, torch, dev, 8, args.scale)
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cpu_sample, min(16, os.cpu_count() or 1))
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
