"""GPU parity: the HIP library, called through its C ABI, against the CPU checker, bit for bit.

Sizes here are ones the checker finishes in seconds; they still span many tiles (a tile is
about a thousand entries) and ragged tails.  Full-size cases are in test_gpu_fullsize.py.
"""
import numpy as np
import pytest
import torch

import brute
from brute import PUT, TOMBSTONE
from gpu_util import as_bytes, assert_probe_equal, build_tree, compact_gpu, dev, probe_gpu, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def g():
    import paper_2511_16138_amd as lsmgpu
    lsmgpu.binding._load()  # raises if the HIP library has not been built
    assert torch.cuda.is_available()
    return lsmgpu


@pytest.fixture(scope="module")
def cfg1():
    from workloads import lsm
    return lsm.config1(device=dev())


def _check_compact(g, oracle, runs, flags):
    got = compact_gpu(g, runs, flags)
    want = oracle.compact([r.cpu() for r in runs], flags & 1)
    assert got.shape[0] == want.shape[0]
    assert np.array_equal(as_bytes(got).reshape(-1, 64), want)
    return got


# ------------------------------------------------------------------ compaction
@pytest.mark.parametrize("flags", [0, 1])
def test_config1_compaction(g, oracle, cfg1, flags):
    print("config1 compaction flags", flags, flush=True)
    _check_compact(g, oracle, cfg1.runs, flags)


def test_generator_is_identical_on_cpu_and_gpu(cfg1):
    from workloads import lsm
    w = lsm.config1(device="cpu")
    assert all(torch.equal(a.cpu(), b) for a, b in zip(cfg1.runs, w.runs))


@pytest.mark.parametrize("scale,flags", [(256, 1), (256, 0), (64, 1), (12, 1)])  # scale 12: 5.6M entries, the sampled partition
def test_scaled_config3_tiered_16way(g, oracle, scale, flags):
    from workloads import lsm
    print("config3 scale", scale, "flags", flags, flush=True)
    w = lsm.config3(device=dev(), scale=scale)
    _check_compact(g, oracle, w.runs, flags)


@pytest.mark.parametrize("flags", [0, 1])
def test_scaled_config2_leveled_two_way(g, oracle, flags):
    from workloads import lsm
    print("config2 scale 50 flags", flags, flush=True)
    w = lsm.config2(device=dev(), scale=50)  # 40,000 + 400,000 entries
    _check_compact(g, oracle, w.runs, flags)


@pytest.mark.parametrize("k", [1, 2, 3, 5, 7, 16, 17, 33, 64])
def test_run_counts_and_ragged_lengths(g, oracle, k):
    """Any run count up to the maximum, uneven and empty runs, lengths that are not tile multiples."""
    from workloads import lsm
    print("ragged k", k, flush=True)
    w = lsm.config3(device=dev(), scale=1024)  # 16 runs x 4096
    rs = np.random.RandomState(k)
    runs = []
    for j in range(k):
        src = w.runs[j % 16]
        n = int(rs.choice([0, 1, 7, 959, 960, 961, 1024, 2500, 4096]))
        start = int(rs.randint(0, 4096 - n + 1))
        r = src[start:start + n].clone()
        r[:, 4] = r[:, 4] ^ (j * 0x9E3779B1)  # different versions in different runs
        runs.append(r)
    for flags in (0, 1):
        _check_compact(g, oracle, runs, flags)


@pytest.mark.parametrize("case", ["same_keys", "interleaved", "one_inside_the_other", "short_and_long", "batch"])
def test_two_runs_many_tiles(g, oracle, case):
    """Two runs (boundaries by bisection on the merge path): every key in both runs (each boundary falls between the
    two versions of some key), keys that alternate between the runs, one run's key range inside the other's, a short
    run against a long one, and the same pairs as jobs of a batch - dozens of tiles each, both flags."""
    from workloads import lsm
    print("two runs", case, flush=True)
    w = lsm.config3(device=dev(), scale=64)           # runs of 65,536 entries
    base = torch.from_numpy(oracle.compact([w.runs[0].cpu(), w.runs[1].cpu()], 0).view(np.int64).reshape(-1, 8).copy()).to(dev())
    older = base.clone()
    older[:, 4] = older[:, 4] - 1                     # the same keys with smaller seqnos
    if case == "same_keys":
        pairs = [(base[:60_000], older[:60_000])]
    elif case == "interleaved":
        pairs = [(base[0:100_000:2].contiguous(), older[1:100_000:2].contiguous())]
    elif case == "one_inside_the_other":
        pairs = [(base[30_000:50_000].contiguous(), older[:90_000].contiguous()), (older[:90_000].contiguous(), base[30_000:50_000].contiguous())]
    elif case == "short_and_long":
        pairs = [(base[77:78].contiguous(), older[:70_000].contiguous()), (base[:70_000].contiguous(), older[5_000:5_003].contiguous())]
    else:
        pairs = [(base[:9_000].contiguous(), older[:9_000].contiguous()), (base[0:30_000:2].contiguous(), older[1:30_000:2].contiguous()),
                 (base[100:101].contiguous(), older[:5_000].contiguous())]
    for flags in (0, 1):
        if case == "batch":
            outs, n_out = g.lsm_compact_batch([(list(p), flags) for p in pairs])
            torch.cuda.synchronize()
            for p, out, n in zip(pairs, outs, n_out.cpu().tolist()):
                want = oracle.compact([r.cpu() for r in p], flags & 1)
                assert n == want.shape[0] and np.array_equal(as_bytes(out[:n]).reshape(-1, 64), want)
        else:
            for p in pairs:
                _check_compact(g, oracle, list(p), flags)


def test_degenerate_inputs(g, oracle):
    from workloads import lsm
    print("degenerate inputs", flush=True)
    w = lsm.config3(device=dev(), scale=1024)
    a = w.runs[0]
    empty = a[:0]
    assert compact_gpu(g, [empty], 1).shape[0] == 0
    assert compact_gpu(g, [empty, empty, empty], 0).shape[0] == 0
    _check_compact(g, oracle, [empty, a[:5], empty], 0)
    _check_compact(g, oracle, [a], 1)  # single run: tombstone filter
    _check_compact(g, oracle, [a], 0)  # single run: copy
    # k identical key sets: the run with the largest seqnos survives whole
    runs = []
    for j, base in enumerate([300, 900, 100, 500]):
        r = a.clone()
        r[:, 4] = base * 100000 + torch.arange(a.shape[0], device=a.device)
        r[:, 6] = j
        runs.append(r)
    got = _check_compact(g, oracle, runs, 0)
    assert bool((got[:, 6] == 1).all())
    # all tombstones into the last level: nothing survives
    t = a.clone()
    t[:, 5] = 1
    assert compact_gpu(g, [t, t[:100].clone()], 1).shape[0] == 0
    # equal seqnos: lowest run index wins
    r0, r1 = a.clone(), a.clone()
    r0[:, 6], r1[:, 6] = 111, 222
    got = _check_compact(g, oracle, [r0, r1], 0)
    assert bool((got[:, 6] == 111).all())
    # disjoint key ranges given in the "wrong" order: concatenation
    _check_compact(g, oracle, [a[3000:], a[:1000], a[1000:3000]], 0)


def test_adversarial_keys_long_common_prefixes(g, oracle):
    """Keys that differ only in their last bytes, and heavy duplication across runs."""
    print("adversarial keys", flush=True)
    rs = np.random.RandomState(77)
    runs = []
    for j in range(6):
        codes = np.unique(rs.randint(0, 6000, size=4000))
        raws = []
        for c in codes:
            key = b"\xAB" * 29 + bytes([(c >> 16) & 0xFF, (c >> 8) & 0xFF, c & 0xFF])
            raws.append(brute.pack_entry(key, int(rs.randint(0, 1 << 62)), TOMBSTONE if rs.rand() < 0.2 else PUT,
                                         vptr=int(rs.randint(1 << 60)), vlen=j, pad0=bytes([j] * 7), pad1=j))
        runs.append(to_dev(brute.run_from_raw(raws)))
    for flags in (0, 1):
        _check_compact(g, oracle, runs, flags)


@pytest.mark.parametrize("n_runs,n_heads,long_groups", [(5, 3000, 0), (16, 1500, 0), (4, 2500, 6)])
def test_keys_that_tie_in_their_first_14_bytes(g, oracle, n_runs, n_heads, long_groups):
    """Small groups of keys equal in the bytes the merge orders by and different after them; with
    long_groups some groups are longer than the in-place repair handles."""
    print("prefix-tie groups", n_runs, n_heads, long_groups, flush=True)
    rs = np.random.RandomState(1000 + n_runs)
    runs = [to_dev(brute.run_from_raw(r)) for r in brute.tie_group_runs(rs, n_runs, n_heads, long_groups)]
    for flags in (0, 1):
        _check_compact(g, oracle, runs, flags)


@pytest.mark.parametrize("separate", [False, True])
def test_first_key_words_that_differ_in_one_bit(g, oracle, separate):
    """Two first key words that differ in their last bit next to one far away (any scaled or
    shortened form of the first word confuses the close pair), mixed inside every run or
    kept in separate runs; the rest of the key is random."""
    print("close first words, separate =", separate, flush=True)
    rs = np.random.RandomState(31 + separate)
    runs = [to_dev(brute.run_from_raw(r)) for r in brute.close_first_words_runs(rs, 6, 1500, separate)]
    for flags in (0, 1):
        _check_compact(g, oracle, runs, flags)


def test_results_do_not_depend_on_repetition(g, cfg1):
    print("determinism", flush=True)
    first = compact_gpu(g, cfg1.runs, 1).clone()
    for _ in range(5):
        assert torch.equal(compact_gpu(g, cfg1.runs, 1), first)


def test_compaction_is_associative_on_gpu(g, oracle, cfg1):
    print("associativity", flush=True)
    newest_first = cfg1.runs
    inner = compact_gpu(g, newest_first[2:], 0).contiguous()        # the two oldest runs
    nested = compact_gpu(g, [newest_first[0], newest_first[1], inner], 1)
    flat = compact_gpu(g, newest_first, 1)
    assert torch.equal(nested, flat)


def test_validate_flag(g, cfg1):
    print("validate", flush=True)
    a = cfg1.runs[0].clone()
    out, n_out = g.lsm_compact([a, cfg1.runs[1]], g.LSM_VALIDATE)
    assert int(n_out.item()) > 0
    bad = a.clone()
    bad[[10, 11]] = bad[[11, 10]]
    with pytest.raises(g.LsmError) as e:
        g.lsm_compact([bad, cfg1.runs[1]], g.LSM_VALIDATE)
    assert e.value.code == -5
    bad = a.clone()
    bad[5, 5] = 7
    with pytest.raises(g.LsmError) as e:
        g.lsm_compact([cfg1.runs[1], bad], g.LSM_VALIDATE)
    assert e.value.code == -6
    small = torch.empty((10, 8), dtype=torch.int64, device=a.device)
    with pytest.raises(g.LsmError) as e:
        g.lsm_compact([a], 0, out=small)
    assert e.value.code == -3


# ------------------------------------------------------------------ fences
@pytest.mark.parametrize("stride", [1, 3, 64, 100, 16383, 16384, 100000])
def test_fences(g, oracle, cfg1, stride):
    print("fences stride", stride, flush=True)
    run = cfg1.runs[0]
    f = g.lsm_build_fences(run, stride)
    torch.cuda.synchronize()
    assert np.array_equal(as_bytes(f).reshape(-1, 32), oracle.build_fences(run.cpu(), stride))


# ------------------------------------------------------------------ probe
def test_config1_probe_before_and_after_compaction(g, oracle, cfg1):
    from workloads import lsm
    print("config1 probe", flush=True)
    q, nb = lsm.queries_config1(cfg1, 4096)
    runs_cpu = [r.cpu() for r in cfg1.runs]
    want = oracle.probe(q, nb, runs_cpu)
    got = probe_gpu(g, q, nb, build_tree(g, cfg1.runs))
    assert_probe_equal(oracle, got, want)
    assert 0.05 < float((want[0] == 0).mean()) < 0.6 and want[0].max() > 32
    for flags in (0, 1):
        merged = compact_gpu(g, cfg1.runs, flags).contiguous()
        got2 = probe_gpu(g, q, nb, build_tree(g, [merged]))
        assert_probe_equal(oracle, got2, oracle.probe(q, nb, [merged.cpu()]))
        assert np.array_equal(got2[0], got[0])                      # same prefix lengths
        assert np.array_equal(got2[1][..., 0], got[1][..., 0])      # same pointers
        assert np.array_equal(got2[1][..., 1] & 0xFFFFFFFF, got[1][..., 1] & 0xFFFFFFFF)  # same lengths


@pytest.mark.parametrize("stride", [1, 7, 64, 1000])
def test_probe_fence_strides_and_row_pitches(g, oracle, cfg1, stride):
    from workloads import lsm
    print("probe stride", stride, flush=True)
    q, nb = lsm.make_queries(cfg1.universe, 300, 1, 100, 0.6, 0.3, None, stream=5, row_blocks=100)
    want = oracle.probe(q, nb, [r.cpu() for r in cfg1.runs])
    assert_probe_equal(oracle, probe_gpu(g, q, nb, build_tree(g, cfg1.runs, stride)), want)


def test_probe_holes_absent_keys_and_edges(g, oracle):
    """A hole ends the prefix even if later blocks are present; keys between, below and above
    the stored keys miss; tombstoned keys are not live; repeated keys are fine."""
    print("probe holes", flush=True)
    rs = np.random.RandomState(21)
    runs_raw = brute.random_runs(rs, 5, 400, 3000, (30, 31), tomb_p=0.25)
    runs = [to_dev(brute.run_from_raw(r)) for r in runs_raw]
    present = sorted({r[:32] for run in runs_raw for r in run})
    requests = []
    for _ in range(600):
        n = int(rs.randint(0, 41))
        req = []
        for _ in range(n):
            u = rs.rand()
            if u < 0.8:
                req.append(present[int(rs.randint(len(present)))])
            elif u < 0.9:
                k = bytearray(present[int(rs.randint(len(present)))]); k[29] = 1; req.append(bytes(k))
            else:
                req.append(bytes(rs.randint(0, 256, size=32).astype(np.uint8)))
        requests.append(req)
    requests += [[b"\x00" * 32], [b"\xff" * 32], []]
    q = np.zeros((len(requests), 40, 32), dtype=np.uint8)
    nb = np.zeros(len(requests), dtype=np.int32)
    for i, req in enumerate(requests):
        nb[i] = len(req)
        for j, k in enumerate(req):
            q[i, j] = np.frombuffer(k, dtype=np.uint8)
    qd = torch.from_numpy(q.view(np.int64).reshape(len(requests), 40, 4).copy()).to(dev())
    nbd = torch.from_numpy(nb).to(dev())
    # random_runs draws seqnos at random; the tree precondition wants newer runs to hold larger ones
    ordered = []
    for j, r in enumerate(runs):
        r = r.clone(); r[:, 4] = (len(runs) - j) * (1 << 40) + (r[:, 4] & 0xFFFFF); ordered.append(r)
    want = oracle.probe(q, nb.astype(np.uint32), [r.cpu() for r in ordered])
    assert_probe_equal(oracle, probe_gpu(g, qd, nbd, build_tree(g, ordered)), want)
    assert (want[0] > 3).any() and (want[0] == 0).any()


def test_probe_empty_tree_and_empty_runs(g, oracle, cfg1):
    from workloads import lsm
    print("probe empty", flush=True)
    q, nb = lsm.queries_config1(cfg1, 64)
    hl, hits = probe_gpu(g, q, nb, [])
    assert (hl == 0).all() and (hits == 0).all()
    empty = cfg1.runs[0][:0]
    tree = build_tree(g, [empty, cfg1.runs[3], empty])
    want = oracle.probe(q, nb, [empty.cpu(), cfg1.runs[3].cpu(), empty.cpu()])
    assert_probe_equal(oracle, probe_gpu(g, q, nb, tree), want)


# ------------------------------------------------------------------ Bloom filters
@pytest.mark.parametrize("bits_per_key", [8, 16])
def test_bloom_filter_bytes_equal_the_checker(g, oracle, cfg1, bits_per_key):
    print("bloom filter", bits_per_key, flush=True)
    for run in list(cfg1.runs) + [cfg1.runs[0][:0], cfg1.runs[1][:1], cfg1.runs[2][:1000]]:
        n_blocks = g.lsm_bloom_blocks(int(run.shape[0]), bits_per_key)
        assert n_blocks == oracle.bloom_blocks(int(run.shape[0]), bits_per_key)
        got = g.lsm_build_bloom(run.contiguous(), bits_per_key)
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(got).reshape(-1, 16), oracle.build_bloom(run.cpu(), n_blocks))
        # building again into the same buffer clears it first
        again = g.lsm_build_bloom(run.contiguous(), bits_per_key, out=got.fill_(-1))
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(again).reshape(-1, 16), oracle.build_bloom(run.cpu(), n_blocks))


def test_probe_with_bloom_filters_gives_the_same_answers(g, oracle, cfg1):
    """Filters only let the probe skip runs that cannot hold a key: results equal the checker's (which
    has no filters) with filters on every run, on some runs, and with a deliberately tiny filter."""
    from workloads import lsm
    print("probe with bloom filters", flush=True)
    q, nb = lsm.queries_config1(cfg1, 2048)
    want = oracle.probe(q, nb, [r.cpu() for r in cfg1.runs])
    plain = build_tree(g, cfg1.runs)
    for choice in ("all", "some", "tiny"):
        tree = []
        for i, t in enumerate(plain):
            bloom = None
            if choice == "all" or (choice == "some" and i % 2 == 0):
                bloom = g.lsm_build_bloom(t.run, 16)
            elif choice == "tiny":
                bloom = g.lsm_build_bloom(t.run, 16, out=torch.empty((3, 4), dtype=torch.int32, device=dev()))  # nearly all ones
            tree.append(g.TreeRun(t.run, t.fences, t.stride, t.level, bloom))
        assert_probe_equal(oracle, probe_gpu(g, q, nb, tree), want)


# ------------------------------------------------------------------ hash index (section 2.2: in-memory indices of a run)
@pytest.mark.parametrize("n", [0, 1, 3, 9, 4096, 16384, 300_000, 65_536 * 5 + 123])
def test_hash_index_is_a_valid_index_of_the_run(g, oracle, n):
    """lsm_build_hash_index: the table passes the checker's validity check (every key in its bucket with its tag and
    position, or its bucket marked crowded and holding seven; nothing else in the table), whatever the buffers held
    before; the key hashes equal the checker's.  The table itself is not unique, so its bytes are not compared."""
    from workloads import lsm
    print("hash index", n, flush=True)
    w = lsm.config3(device=dev(), scale=64)      # 16 runs x 65,536 entries
    run = w.runs[0][:n].contiguous() if n <= 65_536 else torch.cat(list(w.runs))[:n].contiguous()
    if n > 65_536:   # several runs put together are not sorted and hold a key more than once: one sorted run
        cpu = oracle.compact([r.cpu() for r in w.runs], 0)[:n]
        run = torch.from_numpy(cpu.view(np.int64).reshape(-1, 8).copy()).to(dev())
    n = int(run.shape[0])
    hashes = g.lsm_hash_keys(run)
    torch.cuda.synchronize()
    assert np.array_equal(hashes.cpu().numpy().view(np.uint64), oracle.key_hashes(run.cpu()))
    n_buckets = g.lsm_hash_index_buckets(n)
    assert n_buckets == oracle.hash_index_buckets(n)
    table = g.lsm_build_hash_index(hashes, out=torch.full((n_buckets, 8), 0x5A5A5A5A, dtype=torch.int64, device=dev()))
    torch.cuda.synchronize()
    assert oracle.hash_index_check(run.cpu(), table.cpu().numpy()) == 0
    if n >= 4096:
        marks = int(((table[:, 0] >> 15) & 1).sum().item())   # bit 15 of the first tag field
        assert 0 < marks < n_buckets // 10          # some buckets are crowded, most are not


def test_probe_with_hash_indices_gives_the_same_answers(g, oracle, cfg1):
    """A hash index only tells the probe where to look: results equal the checker's (which has none) with an index on
    every run (no fence table in the kernel) or on some, with and without filters, and for the search over the prefix
    length.  Requests made of a run's own keys reach every key of every crowded bucket (the fence path behind the
    mark)."""
    from workloads import lsm
    print("probe with hash indices", flush=True)
    q, nb = lsm.queries_config1(cfg1, 2048)
    runs_cpu = [r.cpu() for r in cfg1.runs]
    want = oracle.probe(q, nb, runs_cpu)
    plain = build_tree(g, cfg1.runs)
    indices = [g.lsm_build_hash_index(g.lsm_hash_keys(t.run)) for t in plain]
    for choice in ("all", "some", "all+filters", "some+filters"):
        tree = []
        for i, t in enumerate(plain):
            index = indices[i] if (not choice.startswith("some") or i % 2 == 0) else None
            bloom = g.lsm_build_bloom(t.run, 16) if choice.endswith("filters") else None
            tree.append(g.TreeRun(t.run, t.fences, t.stride, t.level, bloom, index))
        assert_probe_equal(oracle, probe_gpu(g, q, nb, tree), want)
        got_len = g.lsm_probe_length(q, nb, tree)
        torch.cuda.synchronize()
        assert np.array_equal(got_len.cpu().numpy().astype(np.uint32), want[0])
    # every key of the oldest run as a request of its own row of keys
    run = cfg1.runs[-1]
    n = int(run.shape[0]) // 256 * 256
    own_q = run[:n, :4].reshape(-1, 256, 4).contiguous()
    own_nb = torch.full((own_q.shape[0],), 256, dtype=torch.int32, device=dev())
    want_own = oracle.probe(own_q, own_nb, runs_cpu)
    for tree in ([g.TreeRun(t.run, t.fences, t.stride, t.level, None, ix) for t, ix in zip(plain, indices)],
                 [g.TreeRun(t.run, t.fences, t.stride, t.level, None, ix if i != 1 else None) for i, (t, ix) in enumerate(zip(plain, indices))]):
        assert_probe_equal(oracle, probe_gpu(g, own_q, own_nb, tree), want_own)
    # a table that does not belong to the run (positions far beyond it) must not send a read outside the run
    wrong = torch.full_like(indices[0], (2_000_000_000 << 32) | 2_000_000_000)   # every tag field set, positions beyond the run
    tree = [g.TreeRun(t.run, t.fences, t.stride, t.level, None, wrong if t.run.shape[0] == plain[0].run.shape[0] else None) for t in plain]
    hl, _ = probe_gpu(g, q, nb, tree)
    assert hl.shape == want[0].shape   # the answers are meaningless, the call must simply stay inside the runs


# ------------------------------------------------------------------ pointer rewrite during compaction (section 3.4)
def test_compaction_with_pointer_rewrite(g, oracle, cfg1):
    """lsm_compact_remap = compaction followed by the checker's pointer rewrite: several tensor files folded into
    fewer, files outside the table and tombstones untouched; an empty table is plain compaction."""
    print("pointer rewrite", flush=True)
    runs = cfg1.runs
    files = torch.cat([(r[:, 6] >> 32) & 0xFFFFFFFF for r in runs])
    n_files = int(files.max().item()) + 1
    assert n_files > 4
    table_len = n_files - 2  # the two highest file ids stay as they are
    rs = np.random.RandomState(9)
    # old files f -> new file f // 4, placed one after the other inside it
    starts = rs.randint(0, 1 << 20, size=table_len).cumsum()
    base = torch.tensor([((f // 4) << 32) + int(starts[f]) for f in range(table_len)], dtype=torch.int64, device=dev())
    for flags in (0, 1):
        out, n_out = g.lsm_compact(runs, flags, remap=base)
        torch.cuda.synchronize()
        got = out[: int(n_out.item())]
        plain = oracle.compact([r.cpu() for r in runs], flags & 1)
        want = oracle.remap_pointers(plain, base.cpu().numpy().astype(np.uint64))
        assert np.array_equal(as_bytes(got).reshape(-1, 64), want)
        assert not np.array_equal(want, plain)
        out2, n2 = g.lsm_compact(runs, flags, remap=base[:0])
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(out2[: int(n2.item())]).reshape(-1, 64), plain)


@pytest.mark.parametrize("stride", [1, 64, 100])
def test_fence_index_written_by_the_compaction(g, oracle, cfg1, stride):
    """The fence keys lsm_compact writes along with the run equal those lsm_build_fences and the checker give."""
    print("fused fences", stride, flush=True)
    total = sum(int(r.shape[0]) for r in cfg1.runs)
    for flags in (0, 1):
        fences = torch.full(((total + stride - 1) // stride, 4), -1, dtype=torch.int64, device=dev())
        out, n_out = g.lsm_compact(cfg1.runs, flags, fences=fences, fence_stride=stride)
        torch.cuda.synchronize()
        n = int(n_out.item())
        want = oracle.build_fences(oracle.compact([r.cpu() for r in cfg1.runs], flags & 1), stride)
        n_f = (n + stride - 1) // stride
        assert np.array_equal(as_bytes(fences[:n_f]).reshape(-1, 32), want)
        assert bool((fences[n_f:] == -1).all())  # nothing written past the end


@pytest.mark.parametrize("case", ["cfg1", "one_tile", "empty", "sampled"])
def test_filter_hashes_written_by_the_compaction(g, oracle, cfg1, case):
    """The key hashes lsm_compact writes along with the run are those lsm_hash_keys gives for the merged run, and the
    filter lsm_build_bloom_hashed builds from them is byte for byte the checker's filter of the merged run (so also
    lsm_build_bloom's); fences asked for in the same call are written as well."""
    from workloads import lsm
    print("key hashes from the compaction", case, flush=True)
    if case == "cfg1":
        runs = list(cfg1.runs)
    elif case == "one_tile":
        runs = [cfg1.runs[0][:700].contiguous(), cfg1.runs[1][:300].contiguous()]
    elif case == "empty":
        runs = [cfg1.runs[0][:0].contiguous()]
    else:
        runs = lsm.config3(device=dev(), scale=12).runs   # 5.6M entries: the sampled partition, thousands of tiles
    total = sum(int(r.shape[0]) for r in runs)
    for flags, bits in ((1, 16), (0, 7)):
        hashes = torch.full((max(total, 1),), -1, dtype=torch.int64, device=dev())
        fences = torch.full(((max(total, 1) + 63) // 64, 4), -1, dtype=torch.int64, device=dev()) if flags else None
        out, n_out = g.lsm_compact(runs, flags, key_hashes=hashes, fences=fences, fence_stride=64)
        torch.cuda.synchronize()
        n = int(n_out.item())
        want = oracle.compact([r.cpu() for r in runs], flags & 1)
        assert n == want.shape[0] and np.array_equal(as_bytes(out[:n]).reshape(-1, 64), want)
        assert torch.equal(hashes[:n], g.lsm_hash_keys(out[:n]))
        assert bool((hashes[n:] == -1).all())   # nothing written past the end
        n_blocks = g.lsm_bloom_blocks(n, bits)
        assert n_blocks == oracle.bloom_blocks(n, bits)
        bloom = g.lsm_build_bloom_hashed(hashes[:n], n_blocks, out=torch.full((n_blocks, 4), -1, dtype=torch.int32, device=dev()))
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(bloom).reshape(-1, 16), oracle.build_bloom(want, n_blocks))
        assert torch.equal(bloom, g.lsm_build_bloom(out[:n], bits))
        if fences is not None:
            assert np.array_equal(as_bytes(fences[:(n + 63) // 64]).reshape(-1, 32), oracle.build_fences(want, 64))
    if case == "cfg1":   # the entry point that allocates nothing takes the same request
        out = torch.empty((total, 8), dtype=torch.int64, device=dev())
        n_out = torch.zeros(1, dtype=torch.int64, device=dev())
        hashes = torch.full((total,), -1, dtype=torch.int64, device=dev())
        g.lsm_compact_static(runs, 1, out, n_out, key_hashes=hashes)
        torch.cuda.synchronize()
        n = int(n_out.item())
        assert torch.equal(hashes[:n], g.lsm_hash_keys(out[:n]))


@pytest.mark.parametrize("n,bits", [(0, 16), (1, 16), (5000, 16), (40_000, 16), (300_000, 16), (300_000, 3), (65_536 * 3 + 17, 10)])
def test_filter_built_from_hashes_equals_the_checker(g, oracle, n, bits):
    """lsm_hash_keys + lsm_build_bloom_hashed on runs from one bucket's worth to several chunks and dozens of buckets:
    the same bytes as the checker's filter, whatever the buffers held before; a filter with more blocks than the key
    count asks for (as a caller who sizes it from an upper bound would pass) as well."""
    from workloads import lsm
    print("hashed bloom", n, bits, flush=True)
    w = lsm.config3(device=dev(), scale=64)      # 16 runs x 65,536 entries
    run = torch.cat([r for r in w.runs])[:n].contiguous()   # not sorted across runs: a filter does not care
    for n_blocks in (g.lsm_bloom_blocks(n, bits), g.lsm_bloom_blocks(n, bits) * 3 + 5):
        hashes = g.lsm_hash_keys(run)
        ws = torch.full((max(g.lsm_bloom_workspace_bytes(n, n_blocks), 256),), 0xA5, dtype=torch.uint8, device=dev())
        got = g.lsm_build_bloom_hashed(hashes, n_blocks, out=torch.full((n_blocks, 4), -1, dtype=torch.int32, device=dev()), workspace=ws)
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(got).reshape(-1, 16), oracle.build_bloom(run.cpu(), n_blocks))
    if n == 300_000 and bits == 16:   # a long run with a filter of three blocks: lsm_build_bloom's path for long runs
        tiny = g.lsm_build_bloom(run, 16, out=torch.full((3, 4), -1, dtype=torch.int32, device=dev()))
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(tiny).reshape(-1, 16), oracle.build_bloom(run.cpu(), 3))


# ------------------------------------------------------------------ prefix length by search (appendix B)
def test_probe_length_equals_probe_on_prefix_closed_data(g, oracle, cfg1):
    """The generator evicts leaf first, so its trees are prefix-closed: the search over the prefix length gives the
    checker's first-miss length, with and without Bloom filters, on several runs and on the compacted run."""
    from workloads import lsm
    print("probe length", flush=True)
    q, nb = lsm.queries_config1(cfg1, 4096)
    want = oracle.probe(q, nb, [r.cpu() for r in cfg1.runs])[0]
    tree = build_tree(g, cfg1.runs)
    got = g.lsm_probe_length(q, nb, tree)
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy().astype(np.uint32), want)
    filtered = [g.TreeRun(t.run, t.fences, t.stride, t.level, g.lsm_build_bloom(t.run, 16)) for t in tree]
    assert np.array_equal(g.lsm_probe_length(q, nb, filtered).cpu().numpy().astype(np.uint32), want)
    merged = compact_gpu(g, cfg1.runs, 1).contiguous()
    assert np.array_equal(g.lsm_probe_length(q, nb, build_tree(g, [merged])).cpu().numpy().astype(np.uint32), want)
    # long and short rows, rows of length 0
    nb2 = nb.clone()
    nb2[::7] = 0
    nb2[1::7] = 1
    want2 = oracle.probe(q, nb2, [r.cpu() for r in cfg1.runs])[0]
    assert np.array_equal(g.lsm_probe_length(q, nb2, tree).cpu().numpy().astype(np.uint32), want2)


def test_probe_length_on_data_with_holes(g, oracle):
    """Without prefix closure the result is still a boundary: block j-1 live (or j = 0), block j not (or j = n)."""
    print("probe length with holes", flush=True)
    rs = np.random.RandomState(12)
    keys = sorted({bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(300)})
    present = [k for i, k in enumerate(keys) if rs.rand() < 0.7]
    run = brute.run_from_raw([brute.pack_entry(k, i + 1, TOMBSTONE if rs.rand() < 0.1 else PUT, 1000 + i, 5) for i, k in enumerate(present)])
    live = {brute.unpack(r)[0] for r in brute.raws_of(run) if brute.unpack(r)[2] == PUT}
    n_req, max_blocks = 64, 200
    q = np.zeros((n_req, max_blocks, 32), dtype=np.uint8)
    rows = []
    for r in range(n_req):
        row = [keys[i] for i in rs.choice(len(keys), size=max_blocks, replace=False)]
        rows.append(row)
        q[r] = np.frombuffer(b"".join(row), dtype=np.uint8).reshape(max_blocks, 32)
    nb = rs.randint(0, max_blocks + 1, size=n_req).astype(np.int32)
    qd = torch.from_numpy(q.view(np.int64).reshape(n_req, max_blocks, 4)).to(dev())
    got = g.lsm_probe_length(qd, torch.from_numpy(nb).to(dev()), build_tree(g, [to_dev(run)])).cpu().numpy()
    for r in range(n_req):
        j = int(got[r])
        assert 0 <= j <= nb[r]
        assert j == 0 or rows[r][j - 1] in live
        assert j == nb[r] or rows[r][j] not in live


# ------------------------------------------------------------------ write-buffer flush (section 2.2)
@pytest.mark.parametrize("n,n_keys", [(0, 10), (1, 10), (255, 40), (256, 4000), (3600, 3000), (3600, 50), (8192, 6000),
                                      # beyond 8,192 entries: sorted segments of 4,096, merged by the compaction kernels
                                      (8193, 5000), (10000, 100000), (50000, 40), (100000, 30000), (20000, 10 ** 7),
                                      (262144, 200000)])
def test_flush_of_the_write_buffer(g, oracle, n, n_keys):
    """Unsorted entries with repeated keys and repeated seqnos -> the checker's sorted run, with its fence index."""
    print("flush", n, n_keys, flush=True)
    rs = np.random.RandomState(n + n_keys)
    alphabet = rs.randint(0, 256, size=(n_keys, 32)).astype(np.uint8)
    a = np.zeros((n, 64), dtype=np.uint8)
    if n:
        a[:, :32] = alphabet[rs.randint(0, n_keys, size=n)]
        rec = a.view(oracle.ENTRY_DTYPE).reshape(-1)
        rec["seqno"] = rs.randint(0, 6, size=n) if n_keys <= 50 else rs.randint(0, 1 << 40, size=n)
        rec["type"] = (rs.rand(n) < 0.2).astype(np.uint8)
        rec["vptr"] = np.arange(n)
        rec["vlen"] = 655360
    buf = to_dev(a)
    fences = torch.full(((n + 63) // 64 + 1, 4), -1, dtype=torch.int64, device=dev())
    out, n_out = g.lsm_flush_buffer(buf, fences=fences, fence_stride=64)
    torch.cuda.synchronize()
    want = oracle.flush_buffer(a)
    m = int(n_out.item())
    assert m == want.shape[0]
    assert np.array_equal(as_bytes(out[:m]).reshape(-1, 64), want)
    assert np.array_equal(as_bytes(fences[: (m + 63) // 64]).reshape(-1, 32), oracle.build_fences(want, 64))
    if m:  # a flushed buffer is a run like any other: it compacts and probes
        assert np.array_equal(as_bytes(compact_gpu(g, [out[:m].contiguous()], 0)).reshape(-1, 64), want)


# ------------------------------------------------------------------ range lookups (section 2.2, appendix B get_batch)
def test_range_scan_equals_filtered_compaction(g, oracle, cfg1):
    """Entries of a key range, newest version of each, live only = the checker's last-level compaction of all runs
    cut to the range; one family's range, a range between two stored keys, an empty one and everything."""
    from paper_2511_16138_amd.tree import range_scan
    print("range scan", flush=True)
    tree = build_tree(g, cfg1.runs)
    full = oracle.compact([r.cpu() for r in cfg1.runs], 1)
    keys = [bytes(k) for k in full[:, :32]]
    fam = keys[len(keys) // 3][:8]
    ranges = [(fam + bytes(24), fam + b"\xff" * 24), (keys[100], keys[5000]), (keys[7], keys[7]),
              (bytes(32), b"\xff" * 32), (keys[-1], b"\xff" * 32)]
    for lo, hi in ranges:
        want = full[[i for i, k in enumerate(keys) if lo <= k < hi]] if lo < hi else full[:0]
        bounds = g.lsm_range_bounds(tree, lo, hi).cpu().numpy()
        for (a, b), r in zip(bounds, cfg1.runs):  # every bound is the lower bound of its key in its run
            rk = as_bytes(r).reshape(-1, 64)[:, :32]
            for at, key in ((int(a), lo), (int(b), hi)):
                assert (at == 0 or bytes(rk[at - 1]) < key) and (at == r.shape[0] or bytes(rk[at]) >= key)
        got = range_scan(tree, lo, hi)
        torch.cuda.synchronize()
        assert np.array_equal(as_bytes(got).reshape(-1, 64), want)


def _keys_tensor(keys):
    a = np.frombuffer(b"".join(keys), dtype=np.uint8).reshape(-1, 32).copy()
    return torch.from_numpy(a.view(np.int64).reshape(-1, 4)).to(dev())


@pytest.mark.parametrize("which", ["config1", "tiered16"])
def test_batched_range_scans(g, oracle, cfg1, which):
    """Many key ranges in one call (appendix B, get_batch): every range's entries equal the checker's last-level
    compaction of all runs cut to the range - families, ranges between stored keys, single keys, empty and inverted
    ranges, keys outside the tree; ranges too large for their slot or for a tile are reported as overflow."""
    from workloads import lsm
    print("batched range scans", which, flush=True)
    w = cfg1 if which == "config1" else lsm.config3(device=dev(), scale=256)
    tree = build_tree(g, w.runs)
    full = oracle.compact([r.cpu() for r in w.runs], 1)
    keys = [bytes(k) for k in full[:, :32]]
    run_keys = [[bytes(k) for k in as_bytes(r).reshape(-1, 64)[:, :32]] for r in w.runs]
    all_in = sorted({k for rk in run_keys for k in rk})  # every version's key, dead ones too
    rs = np.random.RandomState(11)
    ranges = []
    for i in rs.randint(0, len(keys), size=300):          # the family of a stored key: all keys with the same first 8 bytes
        fam = keys[i][:8]
        ranges.append((fam + bytes(24), fam + b"\xff" * 24))
    for i in rs.randint(0, len(keys) - 300, size=200):    # between two stored keys, a few to a few hundred entries apart
        ranges.append((keys[i], keys[i + int(rs.randint(0, 300))]))
    for i in rs.randint(0, len(all_in), size=100):        # exactly one key, live or not
        k = all_in[i]
        ranges.append((k, (int.from_bytes(k, "big") + 1).to_bytes(32, "big")))
    ranges += [(keys[7], keys[7]), (keys[50], keys[10]), (bytes(32), keys[0]), (keys[-1], b"\xff" * 32),
               (b"\xff" * 32, b"\xff" * 32), (bytes(32), bytes(32))]
    ranges += [(bytes(32), b"\xff" * 32), (keys[0], keys[len(keys) // 2])]   # far more than a tile: overflow
    import bisect
    max_entries = 512
    ent, cnt = g.lsm_range_scan(tree, _keys_tensor([lo for lo, _ in ranges]), _keys_tensor([hi for _, hi in ranges]), max_entries)
    torch.cuda.synchronize()
    cnt = cnt.cpu().numpy()
    got = as_bytes(ent).reshape(len(ranges), max_entries, 64)
    n_over = 0
    for i, (lo, hi) in enumerate(ranges):
        a, b = (bisect.bisect_left(keys, lo), bisect.bisect_left(keys, hi)) if lo < hi else (0, 0)
        in_pieces = sum(bisect.bisect_left(rk, hi) - bisect.bisect_left(rk, lo) for rk in run_keys) if lo < hi else 0
        if b - a > max_entries or in_pieces > 2048:   # more results than the slot, or more entries (all versions) than a tile
            assert cnt[i] == g.binding.LSM_RANGE_OVERFLOW, (i, cnt[i], b - a, in_pieces)
            n_over += 1
        else:
            assert cnt[i] == b - a, (i, cnt[i], b - a)
            assert np.array_equal(got[i, : b - a], full[a:b]), i
    assert 2 <= n_over < len(ranges) // 2   # the two huge ranges and the large families
    # a small slot: ranges with more results than the slot are reported, the others are unchanged
    ent2, cnt2 = g.lsm_range_scan(tree, _keys_tensor([lo for lo, _ in ranges]), _keys_tensor([hi for _, hi in ranges]), 8)
    cnt2 = cnt2.cpu().numpy()
    got2 = as_bytes(ent2).reshape(len(ranges), 8, 64)
    for i, (lo, hi) in enumerate(ranges):
        a, b = (bisect.bisect_left(keys, lo), bisect.bisect_left(keys, hi)) if lo < hi else (0, 0)
        if b - a > 8:
            assert cnt2[i] == g.binding.LSM_RANGE_OVERFLOW
        elif cnt[i] != g.binding.LSM_RANGE_OVERFLOW:
            assert cnt2[i] == b - a and np.array_equal(got2[i, : b - a], full[a:b])
    # the driver's helper: ranges that overflow their slot are redone one by one, so every range has its content
    from paper_2511_16138_amd.tree import range_scan_batch
    pick = [0, 150, 310, 420, 560, len(ranges) - 1]
    parts = range_scan_batch(tree, _keys_tensor([ranges[i][0] for i in pick]), _keys_tensor([ranges[i][1] for i in pick]), 8)
    for i, part in zip(pick, parts):
        lo, hi = ranges[i]
        a, b = (bisect.bisect_left(keys, lo), bisect.bisect_left(keys, hi)) if lo < hi else (0, 0)
        assert np.array_equal(as_bytes(part).reshape(-1, 64), full[a:b]), i
    # an empty tree and an empty batch
    e0, c0 = g.lsm_range_scan([], _keys_tensor([bytes(32)]), _keys_tensor([b"\xff" * 32]), 4)
    assert c0.cpu().tolist() == [0]
    e1, c1 = g.lsm_range_scan(tree, _keys_tensor([bytes(32)])[:0], _keys_tensor([bytes(32)])[:0], 4)
    assert c1.numel() == 0


def test_batch_of_small_compactions(g, oracle, cfg1):
    """Many independent compactions in one call: every job's output and count equal the checker's for that job -
    1 to 9 runs per job, empty runs and empty jobs, both flag values, jobs of one tile and of dozens of tiles."""
    from workloads import lsm
    print("batch of small compactions", flush=True)
    rs = np.random.RandomState(3)
    src = [r for r in cfg1.runs] + [r for r in lsm.config3(device=dev(), scale=128).runs]
    jobs = []
    for j in range(160):
        k = int(rs.randint(1, 10))
        runs = []
        for r in rs.choice(len(src), size=k, replace=False):   # distinct source runs: one version per key per run
            n = int(src[r].shape[0])
            lo = int(rs.randint(0, n))
            ln = int(rs.choice([0, 1, 7, 100, 1000, 3000, 9000]))
            runs.append(src[r][lo:min(n, lo + ln)].contiguous())
        jobs.append((runs, int(rs.randint(0, 2))))
    jobs.append(([src[0][:0].contiguous()], 1))                       # nothing at all
    jobs.append(([src[0][:0].contiguous(), src[1][:5].contiguous()], 0))
    jobs.append(([r.contiguous() for r in cfg1.runs], 0))              # configuration 1 as one job of the batch
    outs, n_out = g.lsm_compact_batch(jobs)
    torch.cuda.synchronize()
    n_out = n_out.cpu().numpy()
    for j, ((runs, flags), out) in enumerate(zip(jobs, outs)):
        want = oracle.compact([r.cpu() for r in runs], flags)
        assert int(n_out[j]) == want.shape[0], (j, int(n_out[j]), want.shape[0])
        assert np.array_equal(as_bytes(out[: want.shape[0]]).reshape(-1, 64), want), j
    # the same batch again into fresh buffers (the workspace of the first call is gone), with fence indices: same
    # result, and every job's fences are the strided keys of its output
    outs2, n_out2, fences = g.lsm_compact_batch(jobs, fence_stride=64)
    torch.cuda.synchronize()
    assert np.array_equal(n_out2.cpu().numpy(), n_out)
    for a, b, m, f in zip(outs, outs2, n_out, fences):
        assert torch.equal(a[: int(m)], b[: int(m)])
        want_f = as_bytes(a[: int(m)]).reshape(-1, 64)[::64, :32]
        assert np.array_equal(as_bytes(f[: (int(m) + 63) // 64]).reshape(-1, 32), want_f)
    assert g.lsm_compact_batch([])[1].numel() == 0


def test_get_batch_under_a_shared_prefix_with_ladder_keys(g, oracle):
    """get_batch (appendix B) on keys in the segment-ladder layout: the cached blocks below a shared prefix of 512 g
    tokens are one tight key range, fetched for many prefixes in one lsm_range_scan - newest versions, no tombstoned
    blocks - and nothing that is not below the prefix."""
    from test_workloads import _prefix_tree_tokens
    from workloads import keys as K
    print("get_batch with ladder keys", flush=True)
    toks = _prefix_tree_tokens(n_seq=120, length=100, seed=21)
    n, length = toks.shape[0], toks.shape[1]
    words = K.chain_keys(toks, "ladder")                                  # [n, L, 4]
    mem = K.key_bytes_words(words.reshape(-1, 4)).numpy().view(np.uint8).reshape(-1, 32)
    uniq, first_at = np.unique(mem.view("V32").reshape(-1), return_index=True)
    keys_all = mem[np.sort(first_at)]                                     # distinct keys, one per cached block
    rs = np.random.RandomState(5)
    runs, seq = [], 1000
    for r in range(3):                                                    # three runs: random subsets, some tombstones, newer = earlier run
        pick = np.sort(rs.choice(keys_all.shape[0], size=keys_all.shape[0] * 2 // 3, replace=False))
        a = np.zeros((pick.shape[0], 64), dtype=np.uint8)
        a[:, :32] = keys_all[pick]
        rec = a.view(oracle.ENTRY_DTYPE).reshape(-1)
        rec["seqno"] = (3 - r) * 1_000_000 + np.arange(pick.shape[0])
        rec["type"] = (rs.rand(pick.shape[0]) < 0.1).astype(np.uint8)
        rec["vptr"] = rec["seqno"] * 16
        rec["vlen"] = 655360
        order = np.argsort(a[:, :32].view("V32").reshape(-1), kind="stable")
        runs.append(a[order])
    full = oracle.compact(runs, 1)
    full_keys = [bytes(k) for k in full[:, :32]]
    tree = build_tree(g, [to_dev(r) for r in runs])
    kb = [bytes(k) for k in mem]
    t = toks.numpy()
    ranges, below = [], []
    for i in range(0, n, 2):
        for grp in (1, 2, 3):
            deep = kb[i * length + 32 * grp]
            ranges.append((deep[:3 * grp] + bytes(32 - 3 * grp), deep[:3 * grp] + b"\xff" * (32 - 3 * grp)))
            below.append({kb[j * length + k] for j in range(n) if (t[j, :32 * grp] == t[i, :32 * grp]).all() for k in range(32 * grp, length)})
    ent, cnt = g.lsm_range_scan(tree, _keys_tensor([lo for lo, _ in ranges]), _keys_tensor([hi for _, hi in ranges]), 1024)
    torch.cuda.synchronize()
    cnt = cnt.cpu().numpy()
    got = as_bytes(ent).reshape(len(ranges), 1024, 64)
    for i, ((lo, hi), sub) in enumerate(zip(ranges, below)):
        want = full[[j for j, k in enumerate(full_keys) if k in sub]]     # live newest versions of the blocks below the prefix
        assert cnt[i] == want.shape[0], (i, cnt[i], want.shape[0])
        assert np.array_equal(got[i, : cnt[i]], want), i
    assert max(cnt) > 100 and min(cnt) > 0


def test_bloom_filters_of_many_runs_in_one_call(g, oracle, cfg1):
    """lsm_build_bloom_batch: every filter is byte for byte the checker's filter of that run (and so lsm_build_bloom's)."""
    print("bloom batch", flush=True)
    rs = np.random.RandomState(8)
    src = [r for r in cfg1.runs]
    runs = []
    for j in range(70):                      # more than one launch's worth of runs, sizes 0 .. 16,384
        r = src[j % len(src)]
        lo = int(rs.randint(0, r.shape[0]))
        runs.append(r[lo:lo + int(rs.choice([0, 1, 9, 300, 5000, 16384]))].contiguous())
    for bits in (16, 5):
        filters = g.lsm_build_bloom_batch(runs, bits)
        torch.cuda.synchronize()
        for r, f in zip(runs, filters):
            assert int(f.shape[0]) == oracle.bloom_blocks(int(r.shape[0]), bits)
            assert np.array_equal(as_bytes(f).reshape(-1, 16), oracle.build_bloom(r.cpu(), int(f.shape[0])))
    one = g.lsm_build_bloom(runs[5], 16)
    assert torch.equal(one, g.lsm_build_bloom_batch(runs, 16)[5])
    assert g.lsm_build_bloom_batch([], 16) == []
