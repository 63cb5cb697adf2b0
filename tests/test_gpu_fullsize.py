"""GPU parity at the full sizes of the configurations, in the launch configuration bench.py times.

The CPU checker is fast enough (tens of millions of entries per second per core on the GPU
box's host) to merge the full inputs, so compaction outputs are compared entry by entry.
Probes against the 100M-entry tree: all 256 batches (the checker's requests split over the host's cores).
The mixed configuration: the whole trace on the 400M-entry tree, every compaction output and every probe batch.
"""
import time
import numpy as np
import pytest
import torch

from gpu_util import as_bytes, assert_probe_equal, build_tree, compact_gpu, dev, oracle_probe_threads, probe_gpu

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2511_16138_amd as lsmgpu
    lsmgpu.binding._load()
    return lsmgpu


def _full_compare(g, oracle, runs, flags):
    got = compact_gpu(g, runs, flags)
    runs_cpu = [oracle.as_run(r.cpu()) for r in runs]
    want = oracle.compact(runs_cpu, flags & 1)
    assert got.shape[0] == want.shape[0]
    got_np = as_bytes(got).reshape(-1, 64)
    step = 1 << 22
    for i in range(0, want.shape[0], step):
        assert np.array_equal(got_np[i:i + step], want[i:i + step]), f"mismatch in rows {i}..{i + step}"
    return got


def test_config2_full_leveled_2m_into_20m(g, oracle):
    from workloads import lsm
    print("config2 full", flush=True)
    w = lsm.config2(device=dev())
    assert [int(r.shape[0]) for r in w.runs] == [2_000_000, 20_000_000]
    _full_compare(g, oracle, w.runs, 0)


def test_config3_full_tiered_16_way(g, oracle):
    from workloads import lsm
    print("config3 full", flush=True)
    w = lsm.config3(device=dev())
    assert [int(r.shape[0]) for r in w.runs] == [4_194_304] * 16
    del w.universe
    torch.cuda.empty_cache()
    got = _full_compare(g, oracle, w.runs, 1)
    ratio = got.shape[0] / (16 * 4_194_304)
    assert 0.66 < ratio < 0.70  # about 0.95 / 1.4 of the inputs survive


def test_config4_full_tree_all_probe_batches(g, oracle, say):
    """5-level, 100M-entry tree; all 256 batches of 4,096 requests (2^20 requests): hit_len and every hit byte.
    Every 16th batch is also run with Bloom filters and through the search over the prefix length."""
    from workloads import lsm
    say("config4 full tree")
    w = lsm.config4(device=dev())
    assert sum(int(r.shape[0]) for r in w.runs) == 100_000_000 and len(w.runs) == 5
    tree = build_tree(g, w.runs)
    runs_cpu = [oracle.as_run(r.cpu()) for r in w.runs]
    for f, r in zip(tree, runs_cpu):  # fence index of every level, sampled rows
        got_f = as_bytes(f.fences).reshape(-1, 32)
        idx = np.unique(np.linspace(0, got_f.shape[0] - 1, 4096).astype(np.int64))
        assert np.array_equal(got_f[idx], r[idx * 64, :32])
    # Bloom filters of every level in full, and the probe must not change with them
    filtered = [g.TreeRun(t.run, t.fences, t.stride, t.level, g.lsm_build_bloom(t.run, 16)) for t in tree]
    torch.cuda.synchronize()
    for t, r in zip(filtered, runs_cpu):
        assert np.array_equal(as_bytes(t.bloom).reshape(-1, 16), oracle.build_bloom(r, int(t.bloom.shape[0])))
        # the build from the keys' hashes (thousands of block ranges on the 90M-entry level) gives the same bytes
        assert torch.equal(g.lsm_build_bloom_hashed(g.lsm_hash_keys(t.run), int(t.bloom.shape[0])), t.bloom)
    # hash indices of every level: valid tables (the 90M-entry level: 22.5M buckets, thousands of bucket ranges)
    indexed, both = [], []
    for t, f, r in zip(tree, filtered, runs_cpu):
        index = g.lsm_build_hash_index(g.lsm_hash_keys(t.run))
        torch.cuda.synchronize()
        assert oracle.hash_index_check(r, index.cpu().numpy()) == 0
        indexed.append(g.TreeRun(t.run, t.fences, t.stride, t.level, None, index))
        both.append(g.TreeRun(t.run, t.fences, t.stride, t.level, f.bloom, index))
    say("  filters and hash indices ok")
    t0, misses, requests = time.time(), 0, 0
    for stream in range(256):
        q, nb = lsm.queries_config4(w, 4096, stream=stream)
        got = probe_gpu(g, q, nb, tree)
        want = oracle_probe_threads(oracle, q, nb, runs_cpu)
        assert_probe_equal(oracle, got, want)
        misses += int((want[0] == 0).sum())
        requests += int(want[0].shape[0])
        if stream % 16 == 0:
            say(f"  batch {stream} ok ({time.time() - t0:.0f} s)")
            assert_probe_equal(oracle, probe_gpu(g, q, nb, filtered), want)
            assert_probe_equal(oracle, probe_gpu(g, q, nb, indexed), want)
            assert_probe_equal(oracle, probe_gpu(g, q, nb, both), want)
            for t in (tree, filtered, both):  # the generator's data is prefix-closed: the search over the length agrees
                assert np.array_equal(g.lsm_probe_length(q, nb, t).cpu().numpy().astype(np.uint32), want[0])
            assert want[0].max() >= 32
    assert requests == 1 << 20 and 0.25 < misses / requests < 0.45


def test_config5_full_mixed_trace_on_400m_tree(oracle, say):
    """The mixed, shifting workload at its stated size: 6 levels, 400M entries, three phases of 2^18 operations with
    read shares 90 / 50 / 10 %, Bloom filters of 16 bits per key, (T, K) searched over T in 2..16.  Compared with the
    plain driver on the CPU checker: every compaction output byte for byte, every probe batch, every log record - for the
    Python driver over the single entry points and for the library's own driver (lsm_driver_*), stepped side by side."""
    from test_gpu_mixed import replay_both
    from workloads import lsm
    say("config5 full: generating")
    t0 = time.time()
    tr = lsm.config5(device=dev())
    sizes = [int(r.shape[0]) for r in tr.workload.runs]
    assert sum(sizes) == 400_000_000 and len(sizes) == 6 and tr.buffer_entries == 3600
    n_flush = sum(1 for e in tr.events if e[0] == "flush")
    n_batches = sum(1 for e in tr.events if e[0] == "probe")
    say(f"  tree {sizes}, {n_flush} flushes, {n_batches} probe batches ({time.time() - t0:.0f} s)")
    assert n_flush > 4000 and n_batches >= 90
    gpu, n_probe = replay_both(oracle, tr, 16, (2, 16), 16, native=True,
                               progress=lambda msg: say(f"  {msg} ({time.time() - t0:.0f} s)"))
    assert n_probe == n_batches
    comp = [e for e in gpu.trace if e[0] == "compact"]
    pol = [(e[1], e[2]) for e in gpu.trace if e[0] == "policy"]
    say("  policy (T, K):", pol, "compactions:", len(comp), "entries merged:", sum(e[3] for e in comp))
    assert len(comp) > 2000 and max(e[3] for e in comp) > 10_000_000    # compactions down to the fourth level
    assert pol[0][1] == 1 and max(k for _, k in pol) > 1, pol            # leveling under reads, more runs under writes
    assert len({t for t, _ in pol}) > 1 or pol[0][0] != 10, pol
