"""CPU-only checks of the GPU library: it loads, exports the declared C ABI, and its host-side
logic (argument validation, workspace sizing, cost model) behaves as include/lsm_index.h says.
No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2511_16138_amd.binding as B
    if not os.path.exists(B.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return B._load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "lsm_index.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lsm_[a-z_]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    names = declared_functions()
    assert {"lsm_compact", "lsm_compact_workspace_bytes", "lsm_build_fences", "lsm_probe", "lsm_strerror",
            "lsm_policy_levels", "lsm_policy_cost", "lsm_policy_choose"} <= set(names)
    for name in names:
        assert hasattr(lib, name), f"{name} is declared in lsm_index.h but not exported"


def test_struct_sizes_match_the_header():
    import paper_2511_16138_amd.binding as B
    assert C.sizeof(B._Run) == 16 and C.sizeof(B._Out) == 48 and C.sizeof(B._Fence) == 24
    assert C.sizeof(B._Bloom) == 16 and C.sizeof(B._TreeRun) == 80 and C.sizeof(B._Queries) == 24 and C.sizeof(B._Hits) == 16
    assert C.sizeof(B._PolicyInput) == 72
    assert C.sizeof(B._DriverEvent) == 72 and C.sizeof(B._DriverConfig) == 88


def test_driver_arguments_are_checked_before_anything_is_allocated(lib):
    import paper_2511_16138_amd.binding as B
    handle = C.c_void_p(123)
    good = dict(buffer_entries=3600, size_ratio=10, runs_per_level=1, window_ops=4096, shift_threshold=0.2, t_min=2, t_max=16,
                page_entries=64.0, filter_fpr=-1.0, fence_stride=64, bloom_bits=16, hash_index_from=0)
    assert lib.lsm_driver_create(None, None, C.byref(handle)) == -1
    assert lib.lsm_driver_create(C.byref(B._DriverConfig(**good)), None, None) == -1
    for field, bad in [("buffer_entries", 0), ("size_ratio", 1), ("runs_per_level", 0), ("window_ops", 0), ("t_min", 1),
                       ("t_max", 1), ("page_entries", 0.0), ("fence_stride", 0)]:
        cfg = B._DriverConfig(**{**good, field: bad})
        assert lib.lsm_driver_create(C.byref(cfg), None, C.byref(handle)) == -2, field
        assert handle.value is None                       # no driver comes back with an error
    for call, args in [(lib.lsm_driver_note_writes, (None, 1)), (lib.lsm_driver_flush, (None, None, 0)),
                       (lib.lsm_driver_flush_unsorted, (None, None, 0)), (lib.lsm_driver_probe, (None, None, None)),
                       (lib.lsm_driver_load_run, (None, 1, None, 0)), (lib.lsm_driver_target, (None, None, None)),
                       (lib.lsm_driver_level, (None, 1, None, None, None)), (lib.lsm_driver_read, (None, None, None, 0))]:
        assert call(*args) == -1
    one = (C.c_void_p * 1)(None)
    assert lib.lsm_driver_flush_many(None, None, None, 0) == 0          # nothing to do
    assert lib.lsm_driver_flush_many(None, None, None, 1) == -1
    assert lib.lsm_driver_flush_many(one, (C.c_void_p * 1)(None), (C.c_uint64 * 1)(0), 1) == -1   # a NULL driver
    assert lib.lsm_driver_levels(None) == 0 and lib.lsm_driver_log(None, 0, None, 0) == 0
    lib.lsm_driver_destroy(None)                          # allowed


def test_argument_errors_are_reported_before_any_launch(lib):
    import paper_2511_16138_amd.binding as B
    n_out = C.c_uint64(123)
    run = B._Run(None, 0)
    out = B._Out(None, 0, C.addressof(n_out), None, 0)
    assert lib.lsm_compact(None, 1, 0, C.byref(out), None, 0, None) == -1          # NULL runs
    assert lib.lsm_compact(C.byref(run), 0, 0, C.byref(out), None, 0, None) == -2  # n_runs == 0
    assert lib.lsm_compact(C.byref(run), 65, 0, C.byref(out), None, 0, None) == -2
    bad = B._Run(None, 5)
    assert lib.lsm_compact(C.byref(bad), 1, 0, C.byref(out), None, 0, None) == -1  # n > 0 but no entries
    fake = B._Run(64 * 1000, 10)
    small = B._Out(64 * 2000, 9, C.addressof(n_out), None, 0)
    assert lib.lsm_compact(C.byref(fake), 1, 0, C.byref(small), None, 0, None) == -3  # capacity
    big = B._Out(64 * 2000, 10, C.addressof(n_out), None, 0)
    assert lib.lsm_compact(C.byref(fake), 1, 0, C.byref(big), None, 0, None) == -4    # workspace
    assert lib.lsm_compact(C.byref(fake), 1, 0, C.byref(big), 256 * 7, 16, None) == -4
    misaligned = B._Run(64 * 1000 + 8, 10)
    assert lib.lsm_compact(C.byref(misaligned), 1, 0, C.byref(big), 256 * 7, 1 << 20, None) == -2
    assert n_out.value == 123
    # new entry points: the same kind of checks, all before any launch
    fenced = B._Out(64 * 2000, 10, C.addressof(n_out), 16 * 5, 0)
    assert lib.lsm_compact(C.byref(fake), 1, 0, C.byref(fenced), 256 * 7, 1 << 20, None) == -2     # fence stride 0
    odd = B._Out(64 * 2000, 10, C.addressof(n_out), 16 * 5 + 4, 64)
    assert lib.lsm_compact(C.byref(fake), 1, 0, C.byref(odd), 256 * 7, 1 << 20, None) == -2        # fence keys misaligned
    hashed = B._Out(64 * 2000, 10, C.addressof(n_out), None, 0, 8 * 7 + 4)
    assert lib.lsm_compact(C.byref(fake), 1, 0, C.byref(hashed), 256 * 7, 1 << 20, None) == -2     # key hashes misaligned
    hashed = B._Out(64 * 2000, 10, C.addressof(n_out), None, 0, 8 * 7)
    assert lib.lsm_flush_buffer(64 * 10, 10, C.byref(hashed), 256, 1 << 20, None) == -2            # a flush writes no hashes
    assert lib.lsm_bloom_workspace_bytes(0, 1) > 0 and lib.lsm_bloom_workspace_bytes(10, 0) == 0
    assert lib.lsm_bloom_workspace_bytes(1 << 32, 1 << 20) == 0 and lib.lsm_bloom_workspace_bytes(10, (1 << 25) + 1) == 0
    assert 8 * 1_000_000 <= lib.lsm_bloom_workspace_bytes(1_000_000, 125_000) < 8 * 1_000_000 + 4096
    assert lib.lsm_build_bloom_hashed(None, 5, 16 * 9, 4, 256 * 3, 1 << 20, None) == -1            # no hashes
    assert lib.lsm_build_bloom_hashed(8 * 3, 5, 16 * 9, 0, 256 * 3, 1 << 20, None) == -2           # no blocks
    assert lib.lsm_build_bloom_hashed(8 * 3, 5, 16 * 9 + 8, 4, 256 * 3, 1 << 20, None) == -2       # filter misaligned
    assert lib.lsm_build_bloom_hashed(8 * 3, 5, 16 * 9, 4, 256 * 3, 16, None) == -4                # workspace too small
    assert lib.lsm_build_bloom_hashed(8 * 3, 5, 16 * 9, 4, 256 * 3 + 8, 1 << 20, None) == -4       # workspace misaligned
    assert lib.lsm_hash_keys(C.byref(fake), None, None) == -1
    assert lib.lsm_hash_keys(C.byref(fake), 8 * 5 + 1, None) == -2
    assert [lib.lsm_hash_index_buckets(n) for n in (0, 1, 4, 5, 1 << 20)] == [1, 1, 1, 2, 1 << 18]
    assert lib.lsm_hash_index_workspace_bytes((1 << 27) + 1) == 0 and lib.lsm_hash_index_workspace_bytes(0) > 0
    assert 16 * 1_000_000 <= lib.lsm_hash_index_workspace_bytes(1_000_000) < 16 * 1_000_000 + 8192
    assert lib.lsm_build_hash_index(None, 5, 64 * 9, 256 * 3, 1 << 20, None) == -1                 # no hashes
    assert lib.lsm_build_hash_index(8 * 3, 5, 64 * 9 + 8, 256 * 3, 1 << 20, None) == -2            # table misaligned
    assert lib.lsm_build_hash_index(8 * 3, (1 << 27) + 1, 64 * 9, 256 * 3, 1 << 40, None) == -2    # run too long
    assert lib.lsm_build_hash_index(8 * 3, 5, 64 * 9, 256 * 3, 16, None) == -4                     # workspace too small
    table = B._Remap(None, 3)
    assert lib.lsm_compact_remap(C.byref(fake), 1, 0, C.byref(big), 256 * 7, 1 << 20, None, C.byref(table), None) == -1
    assert lib.lsm_flush_workspace_bytes(3600) == 14400 and lib.lsm_flush_workspace_bytes(1 << 20) == 0
    assert 64 * 100000 < lib.lsm_flush_workspace_bytes(100000) < 80 * 100000   # sorted segments + merge workspace
    assert lib.lsm_flush_buffer(64 * 10, 300000, C.byref(big), 256, 1 << 20, None) == -2  # too many entries
    assert lib.lsm_flush_buffer(None, 5, C.byref(big), 256, 1 << 20, None) == -1
    assert lib.lsm_flush_buffer(64 * 10, 11, C.byref(big), 256, 1 << 20, None) == -3      # capacity 10
    assert lib.lsm_flush_buffer(64 * 10, 10, C.byref(big), 256, 8, None) == -4            # workspace
    assert lib.lsm_bloom_blocks(0, 16) == 1 and lib.lsm_bloom_blocks(9, 16) == 2 and lib.lsm_bloom_blocks(5, 0) == 0
    assert lib.lsm_bloom_blocks(1 << 40, 16) == 0
    assert lib.lsm_build_bloom(None, 64, 1, None) == -1 and lib.lsm_build_bloom(C.byref(fake), None, 1, None) == -1
    assert lib.lsm_build_bloom(C.byref(fake), 64, 0, None) == -2 and lib.lsm_build_bloom(C.byref(fake), 64 + 8, 1, None) == -2
    assert lib.lsm_build_fences(C.byref(fake), 0, 4096, None) == -2
    assert lib.lsm_build_fences(None, 64, 4096, None) == -1
    assert lib.lsm_build_fences(C.byref(run), 64, None, None) == 0  # empty run: nothing to do
    q = B._Queries(4096, 8192, 4, 257)
    tree = B._Tree(None, 0)
    hits = B._Hits(4096, 8192)
    assert lib.lsm_probe(C.byref(q), C.byref(tree), C.byref(hits), None) == -2  # max_blocks > 256
    q = B._Queries(None, None, 0, 16)
    assert lib.lsm_probe(C.byref(q), C.byref(tree), C.byref(hits), None) == 0   # empty batch
    tr = (B._TreeRun * 1)()
    tr[0].run, tr[0].fence = B._Run(64 * 1000, 100), B._Fence(4096, 1, 64)        # needs 2 fences
    q = B._Queries(4096, 8192, 4, 16)
    assert lib.lsm_probe(C.byref(q), C.byref(B._Tree(tr, 1)), C.byref(hits), None) == -2
    ptrs, nbs = (C.c_void_p * 2)(64, 128), (C.c_uint64 * 2)(4, 0)
    two = (B._Run * 2)(fake, fake)
    assert lib.lsm_build_bloom_batch(two, ptrs, nbs, 2, None) == -2      # a filter of zero blocks
    assert lib.lsm_build_bloom_batch(None, ptrs, nbs, 2, None) == -1 and lib.lsm_build_bloom_batch(None, None, None, 0, None) == 0
    # batched forms: argument errors before any launch
    rg = B._Ranges(4096, 8192, 3, 4096)
    ro = B._RangeOut(64 * 1000, 4096)
    assert lib.lsm_range_scan(C.byref(rg), C.byref(tree), C.byref(ro), None) == -2          # slot larger than a tile
    assert lib.lsm_range_scan(C.byref(B._Ranges(None, None, 3, 16)), C.byref(tree), C.byref(ro), None) == -1
    assert lib.lsm_range_scan(C.byref(B._Ranges(4096 + 8, 8192, 3, 16)), C.byref(tree), C.byref(ro), None) == -2
    assert lib.lsm_range_scan(C.byref(B._Ranges(None, None, 0, 16)), C.byref(tree), C.byref(ro), None) == 0   # no ranges
    job = (B._CompactJob * 1)()
    job[0].runs, job[0].n_runs, job[0].flags, job[0].out = C.pointer(fake), 1, 0, big
    need = lib.lsm_compact_batch_workspace_bytes(job, 1)
    assert need >= 256 * 6
    assert lib.lsm_compact_batch(job, 1, 256 * 7, need - 1, None) == -4
    job[0].flags = 2
    assert lib.lsm_compact_batch_workspace_bytes(job, 1) == 0 and lib.lsm_compact_batch(job, 1, 256 * 7, 1 << 20, None) == -2
    job[0].flags, job[0].out = 0, small
    assert lib.lsm_compact_batch(job, 1, 256 * 7, 1 << 20, None) == -3
    job[0].out, job[0].runs = big, C.pointer(B._Run(64 * 1000, 1 << 23))
    assert lib.lsm_compact_batch(job, 1, 256 * 7, 1 << 30, None) == -2                          # too large for the batch
    assert lib.lsm_compact_batch(None, 0, None, 0, None) == 0
    # the entry point without a workspace argument: same checks, plus its size limit, all before any launch
    assert lib.lsm_compact_static(None, 1, 0, C.byref(out), None) == -1
    assert lib.lsm_compact_static(C.byref(run), 0, 0, C.byref(out), None) == -2
    assert lib.lsm_compact_static(C.byref(fake), 1, 2, C.byref(big), None) == -2      # LSM_VALIDATE needs the host
    huge = B._Run(64 * 1000, 1 << 26)
    assert lib.lsm_compact_static(C.byref(huge), 1, 0, C.byref(big), None) == -9      # beyond the static scratch
    assert n_out.value == 123
    for code in range(-9, 1):
        assert lib.lsm_strerror(code) and lib.lsm_strerror(code) != b"unknown status"
    assert lib.lsm_strerror(-99) == b"unknown status"


def test_workspace_size_is_monotone_and_small(lib):
    import paper_2511_16138_amd as g
    assert g.lsm_compact_workspace_bytes([]) == 0
    a = g.lsm_compact_workspace_bytes([0, 0])
    b = g.lsm_compact_workspace_bytes([1 << 22] * 16)
    assert 256 <= a < b < (1 << 22) * 16 * 64 // 50  # a few percent of the data at most


def test_cost_model_matches_the_checker(lib, oracle):
    import paper_2511_16138_amd as g
    rs = np.random.RandomState(5)
    for _ in range(200):
        w, s, r, z = rs.dirichlet([1, 1, 1, 1])
        N, M = int(rs.randint(1, 1 << 40)), int(rs.randint(1, 1 << 16))
        T = int(rs.randint(2, 17))
        K = int(rs.randint(1, T)) if T > 2 else 1
        B_, p, d = float(rs.choice([16, 64, 256])), float(rs.choice([1.0, 0.1, 0.01])), float(rs.randint(0, 512))
        assert g.lsm_policy_levels(N, M, T) == oracle.levels(N, M, T)
        assert g.lsm_policy_cost(w, s, r, z, N, M, T, K, B_, p, d) == oracle.cost(w, s, r, z, N, M, T, K, B_, p, d)
        assert g.lsm_policy_choose(w, s, r, z, N, M, 2, 16, B_, p, d) == oracle.policy_choose(w, s, r, z, N, M, 2, 16, B_, p, d)
    for T in (2, 10):
        for e in range(1, 15):
            assert g.lsm_policy_levels(T ** e, 1, T) == e and g.lsm_policy_levels(T ** e + 1, 1, T) == e + 1
    assert g.lsm_policy_choose(1, 0, 0, 0, 400_000_000, 3600, 10, 10, 64.0, 1.0, 64.0) == (10, 9)
    assert g.lsm_policy_choose(0, 0.3, 0.3, 0.4, 400_000_000, 3600, 10, 10, 64.0, 1.0, 64.0) == (10, 1)
    with pytest.raises(g.LsmError):
        g.lsm_policy_choose(1, 0, 0, 0, 10, 0, 2, 4, 64.0, 1.0, 0.0)
