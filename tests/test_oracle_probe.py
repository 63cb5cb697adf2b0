"""Pins for the C checker's probe, fence index and cost model (CPU only)."""
import bisect
import os

import numpy as np
import pytest

import brute
from brute import PUT, TOMBSTONE
from test_oracle_compaction import small_key, worked_runs

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _pack_requests(requests, max_blocks):
    q = np.zeros((len(requests), max_blocks, 32), dtype=np.uint8)
    nb = np.zeros(len(requests), dtype=np.uint32)
    for i, req in enumerate(requests):
        nb[i] = len(req)
        for j, k in enumerate(req):
            q[i, j] = np.frombuffer(k, dtype=np.uint8)
    return q, nb


def _op(oracle, runs, requests, max_blocks):
    q, nb = _pack_requests(requests, max_blocks)
    hit_len, hits = oracle.probe(q, nb, [brute.run_from_raw(r) for r in runs])
    rows = [[(int(h["vptr"]), int(h["vlen"]), int(h["run_idx"])) for h in hits[i]] for i in range(len(requests))]
    return [int(x) for x in hit_len], rows


def test_probe_worked_example(oracle):
    raw_runs, _, probes = worked_runs()
    for req, want_len, want_runs in probes:
        hit_len, rows = _op(oracle, raw_runs, [[small_key(k) for k in req]], 8)
        assert hit_len == [want_len]
        assert [r[2] for r in rows[0][:want_len]] == want_runs
        for j in range(want_len):  # pointer of the version found, as packed by worked_runs()
            assert rows[0][j][0] == 1000 * want_runs[j] + req[j] and rows[0][j][1] == 64 + req[j]
        assert all(r == (0, 0, 0) for r in rows[0][want_len:])


@pytest.mark.parametrize("vary", [(31,), (0, 31), (8, 9)])
def test_probe_equals_exhaustive_scan_on_tiny_trees(oracle, vary):
    rs = np.random.RandomState(11 + len(vary))
    for _ in range(120):
        n_runs = int(rs.randint(1, 6))
        runs = brute.random_runs(rs, n_runs, 12, int(rs.choice([6, 30, 120])), vary, tomb_p=0.25)
        present = sorted({r[:32] for run in runs for r in run})
        absent = [bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(4)]
        requests = []
        for _ in range(10):
            n = int(rs.randint(0, 9))
            pool = present + absent if present else absent
            requests.append([pool[int(rs.randint(len(pool)))] for _ in range(n)])  # holes and repeats occur
        assert _op(oracle, runs, requests, 8) == brute.probe(runs, requests, 8)


def test_every_tree_key_alone_is_live_iff_newest_is_put(oracle):
    rs = np.random.RandomState(12)
    runs = brute.random_runs(rs, 4, 60, 150, (30, 31), tomb_p=0.3)
    keys = sorted({r[:32] for run in runs for r in run})
    hit_len, _ = _op(oracle, runs, [[k] for k in keys], 1)
    for k, h in zip(keys, hit_len):
        assert h == (1 if brute.unpack(brute.newest(runs, k)[2])[2] == PUT else 0)


def test_keys_between_below_and_above_entries_miss(oracle):
    keys = [bytes([0] * 30 + [a, 0x80]) for a in range(1, 60)]
    run = [brute.pack_entry(k, i, PUT, vptr=i + 1) for i, k in enumerate(keys)]
    between = [bytes([0] * 30 + [a, 0x81]) for a in range(1, 60)] + [bytes([0] * 30 + [a, 0x7F]) for a in range(1, 60)]
    edges = [b"\x00" * 32, b"\xff" * 32]
    hit_len, _ = _op(oracle, [run[:30], run[30:]], [[k] for k in between + edges], 1)
    assert hit_len == [0] * len(hit_len)
    hit_len, rows = _op(oracle, [run[:30], run[30:]], [[k] for k in keys], 1)
    assert hit_len == [1] * len(keys)
    assert [r[0][0] for r in rows] == list(range(1, 60))  # the pointer of exactly that entry


def test_single_run_single_key_is_binary_search(oracle):
    rs = np.random.RandomState(13)
    keys = sorted({bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(400)})
    run = [brute.pack_entry(k, i, PUT, vptr=i) for i, k in enumerate(keys)]
    qs = [keys[int(rs.randint(len(keys)))] if rs.rand() < 0.5 else bytes(rs.randint(0, 256, size=32).astype(np.uint8))
          for _ in range(300)]
    hit_len, rows = _op(oracle, [run], [[k] for k in qs], 1)
    for k, h, row in zip(qs, hit_len, rows):
        i = bisect.bisect_left(keys, k)
        found = i < len(keys) and keys[i] == k
        assert h == int(found) and (not found or row[0][0] == i)


def test_compaction_preserves_lookups(oracle):
    rs = np.random.RandomState(14)
    for _ in range(40):
        runs = brute.random_runs(rs, 4, 40, 90, (30, 31), tomb_p=0.3)
        keys = sorted({r[:32] for run in runs for r in run})
        requests = [[keys[int(rs.randint(len(keys)))] for _ in range(int(rs.randint(1, 6)))] for _ in range(30)] if keys else []
        before = _op(oracle, runs, requests, 8)
        for bottom in (False, True):
            merged = brute.raws_of(oracle.compact([brute.run_from_raw(r) for r in runs], 1 if bottom else 0))
            after = _op(oracle, [merged], requests, 8)
            assert after[0] == before[0]
            strip = lambda rows: [[(v, l) for v, l, _ in row] for row in rows]
            assert strip(after[1]) == strip(before[1])  # all but run_idx


def test_generated_requests_hit_what_was_inserted(oracle):
    import torch
    from workloads import lsm
    w = lsm.config1()
    runs = [oracle.as_run(r) for r in w.runs]
    q, nb = lsm.queries_config1(w, 512)
    hit_len, hits = oracle.probe(q, nb, runs)
    merged = oracle.compact(runs, 0)
    hit_len2, hits2 = oracle.probe(q, nb, [merged])
    assert np.array_equal(hit_len, hit_len2)
    assert np.array_equal(hits["vptr"], hits2["vptr"]) and np.array_equal(hits["vlen"], hits2["vlen"])
    frac_zero = float((hit_len == 0).mean())
    assert 0.05 < frac_zero < 0.5 and hit_len.max() > 32  # misses and long prefix hits both occur
    # a request whose first block is fresh random tokens can never hit
    qf, nbf = lsm.make_queries(w.universe, 64, 16, 64, 0.0, 0.0, None, stream=9, row_blocks=64)
    assert (oracle.probe(qf, nbf, runs)[0] == 0).all()
    # the tree honours the LSM precondition: for a key in several runs the newer run has the larger seqno
    seen = {}
    for r in reversed(range(len(runs))):
        seq = runs[r][:, 32:40].copy().view("<u8").ravel()
        for i in range(0, runs[r].shape[0], 7):
            k = runs[r][i, :32].tobytes()
            assert seen.get(k, -1) < int(seq[i])
            seen[k] = int(seq[i])



def test_generated_data_is_prefix_closed(oracle):
    """Leaf-first eviction keeps the data prefix-closed: in every generated request the live block keys are exactly
    the first hit_len ones (what makes the search over the prefix length of appendix B valid on these inputs)."""
    from workloads import lsm
    w = lsm.config1()
    runs = [oracle.as_run(r) for r in w.runs]
    live = {bytes(k) for k in oracle.compact(runs, 1)[:, :32]}  # newest version is a PUT
    q, nb = lsm.queries_config1(w, 512)
    hit_len = oracle.probe(q, nb, runs)[0]
    qb = q.numpy().view(np.uint8).reshape(q.shape[0], q.shape[1], 32)
    for r in range(qb.shape[0]):
        flags = [bytes(qb[r, j]) in live for j in range(int(nb[r]))]
        assert flags == [j < hit_len[r] for j in range(int(nb[r]))]


# ---------------------------------------------------------------- fences
def test_fences_are_strided_keys_and_bound_searches(oracle):
    rs = np.random.RandomState(15)
    keys = sorted({bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(1000)})
    run = brute.run_from_raw([brute.pack_entry(k, i, PUT) for i, k in enumerate(keys)])
    for stride in (1, 3, 64, 999, 1000, 5000):
        f = oracle.build_fences(run, stride)
        want = keys[::stride]
        assert [f[i].tobytes() for i in range(f.shape[0])] == want
        assert all(want[i] < want[i + 1] for i in range(len(want) - 1))
        # lower_bound through the fences (page = [i*stride, (i+1)*stride)) equals lower_bound on the run
        for _ in range(200):
            k = keys[int(rs.randint(len(keys)))] if rs.rand() < 0.5 else bytes(rs.randint(0, 256, size=32).astype(np.uint8))
            page = max(0, bisect.bisect_right(want, k) - 1)
            lo, hi = page * stride, min(len(keys), (page + 1) * stride)
            assert lo + bisect.bisect_left(keys[lo:hi], k) == bisect.bisect_left(keys, k)
    assert oracle.build_fences(run[:0], 64).shape == (0, 32)


# ---------------------------------------------------------------- cost model
def test_cost_model_golden_values(oracle):
    rows = 0
    for line in open(os.path.join(GOLDEN, "cost_model.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        lhs, rhs = line.split("->")
        N, M, T, K, B, p, d, w, s, r, z = lhs.split()
        L, W, S, R, Z, total = [float(x) for x in rhs.split()]
        N, M, T, K = int(N), int(M), int(T), int(K)
        B, p, d, w, s, r, z = (float(x) for x in (B, p, d, w, s, r, z))
        assert oracle.levels(N, M, T) == int(L)
        assert oracle.cost(1, 0, 0, 0, N, M, T, K, B, p, d) == pytest.approx(W, rel=1e-13)
        assert oracle.cost(0, 1, 0, 0, N, M, T, K, B, p, d) == pytest.approx(S, rel=1e-13)
        assert oracle.cost(0, 0, 1, 0, N, M, T, K, B, p, d) == pytest.approx(R, rel=1e-13)
        assert oracle.cost(0, 0, 0, 1, N, M, T, K, B, p, d) == pytest.approx(Z, rel=1e-13)
        assert oracle.cost(w, s, r, z, N, M, T, K, B, p, d) == pytest.approx(total, rel=1e-13)
        rows += 1
    assert rows >= 7


def test_policy_extremes_match_the_paper(oracle):
    # section 3.3: write-heavy windows favour tiering (large K), read-heavy ones leveling (K = 1)
    N, M = 400_000_000, 3600
    assert oracle.policy_choose(1.0, 0.0, 0.0, 0.0, N, M, 10, 10, 64.0, 1.0, 64.0) == (10, 9)
    assert oracle.policy_choose(0.0, 0.3, 0.3, 0.4, N, M, 10, 10, 64.0, 1.0, 64.0) == (10, 1)
    # argmin agrees with a scan in Python over the same grid, with the documented tie-break
    rs = np.random.RandomState(16)
    for _ in range(50):
        w, s, r, z = rs.dirichlet([1, 1, 1, 1])
        best = None
        for T in range(2, 17):
            for K in range(1, T):
                c = oracle.cost(w, s, r, z, N, M, T, K, 64.0, 1.0, 64.0)
                if best is None or c < best[0] or (c == best[0] and (K, T) < (best[2], best[1])):
                    best = (c, T, K)
        assert oracle.policy_choose(w, s, r, z, N, M, 2, 16, 64.0, 1.0, 64.0) == (best[1], best[2])
    # L from integer powers, no floating-point log: exact at powers of T
    for T in (2, 3, 10):
        for e in range(1, 12):
            assert oracle.levels(T ** e, 1, T) == e and oracle.levels(T ** e + 1, 1, T) == e + 1
    assert oracle.levels(1, 1000, 10) == 1
