"""Pins for the C checker's key order and compaction (CPU only).

Nothing here calls the GPU library.  The checker is compared with: libc-free Python byte
comparison, a sort+dedup definition written in Python (tests/brute.py), a hand-worked
example (tests/golden), invariants of the result, and special cases that reduce to
sorted()/heapq.merge.
"""
import heapq
import os

import numpy as np
import pytest

import brute
from brute import PUT, TOMBSTONE

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _oc(oracle, runs, bottommost):
    out = oracle.compact([brute.run_from_raw(r) for r in runs], oracle.FLAG_BOTTOMMOST if bottommost else 0)
    return brute.raws_of(out)


# ---------------------------------------------------------------- key order
def test_key_cmp_every_byte_position(oracle):
    base = bytes(range(7, 39))
    for i in range(32):
        lo, hi = bytearray(base), bytearray(base)
        lo[i], hi[i] = 0x10, 0x90  # 0x90 > 0x10 only if bytes compare unsigned
        # make every later byte pull the other way: the first difference must decide
        for j in range(i + 1, 32):
            lo[j], hi[j] = 0xFF, 0x00
        assert oracle.key_cmp(bytes(lo), bytes(hi)) < 0
        assert oracle.key_cmp(bytes(hi), bytes(lo)) > 0
    assert oracle.key_cmp(base, base) == 0
    assert oracle.key_cmp(b"\x00" * 32, b"\xff" * 32) < 0
    assert oracle.key_cmp(b"\x7f" + b"\xff" * 31, b"\x80" + b"\x00" * 31) < 0


def test_key_cmp_matches_python_bytes_order(oracle):
    rs = np.random.RandomState(1)
    for _ in range(2000):
        a = bytearray(rs.randint(0, 4, size=32).astype(np.uint8))
        b = bytearray(a) if rs.rand() < 0.5 else bytearray(rs.randint(0, 4, size=32).astype(np.uint8))
        if rs.rand() < 0.5:
            b[rs.randint(32)] = rs.randint(256)
        a, b = bytes(a), bytes(b)
        got = oracle.key_cmp(a, b)
        assert (got < 0) == (a < b) and (got > 0) == (a > b)


# ---------------------------------------------------------------- hand-worked example
def _parse_items(text):
    items = []
    for tok in text.split():
        k, s, t = tok.split(":")
        items.append((int(k), int(s), PUT if t == "P" else TOMBSTONE))
    return items


def load_worked_example():
    runs, expect, probes = {}, {}, []
    for line in open(os.path.join(GOLDEN, "compaction_worked_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("run "):
            head, rest = line.split(":", 1)
            runs[int(head.split()[1])] = _parse_items(rest)
        elif line.startswith("expect "):
            head, rest = line.split(":", 1)
            expect[head.split()[1]] = _parse_items(rest)
        elif line.startswith("probe "):
            lhs, rhs = line[len("probe "):].split("->")
            words = rhs.split()
            probes.append(([int(x) for x in lhs.split()], int(words[1]), [int(x) for x in words[3:]]))
    return [runs[i] for i in sorted(runs)], expect, probes


def small_key(b: int) -> bytes:
    return b"\x00" * 31 + bytes([b])


def worked_runs():
    runs, expect, probes = load_worked_example()
    raw_runs = [[brute.pack_entry(small_key(k), s, t, vptr=1000 * r + k, vlen=64 + k) for k, s, t in run]
                for r, run in enumerate(runs)]
    return raw_runs, expect, probes


def test_compaction_worked_example(oracle):
    raw_runs, expect, _ = worked_runs()
    for name, bottom in (("keep_tombstones", False), ("bottommost", True)):
        got = [(brute.unpack(r)[0][31], brute.unpack(r)[1], brute.unpack(r)[2]) for r in _oc(oracle, raw_runs, bottom)]
        assert got == expect[name]


# ---------------------------------------------------------------- brute force on tiny inputs
@pytest.mark.parametrize("vary", [(31,), (0,), (7, 8), (15, 16, 31), (0, 31)])
def test_compaction_equals_sort_dedup_on_tiny_inputs(oracle, vary):
    rs = np.random.RandomState(hash(vary) % (1 << 31))
    for trial in range(150):
        n_runs = int(rs.randint(1, 6))
        alphabet = int(rs.choice([3, 8, 40, 200]))
        runs = brute.random_runs(rs, n_runs, 14, alphabet, vary, tomb_p=float(rs.choice([0.0, 0.3, 1.0])),
                                 force_seq_ties=(trial % 5 == 0))
        for bottom in (False, True):
            assert _oc(oracle, runs, bottom) == brute.compact(runs, bottom)


def test_seqno_tie_goes_to_lowest_run_index(oracle):
    k = small_key(5)
    runs = [[brute.pack_entry(k, 7, PUT, vptr=111)], [brute.pack_entry(k, 7, TOMBSTONE, vptr=222)],
            [brute.pack_entry(k, 7, PUT, vptr=333)]]
    out = _oc(oracle, runs, False)
    assert len(out) == 1 and brute.unpack(out[0])[3] == 111
    out = _oc(oracle, runs[1:], False)
    assert brute.unpack(out[0])[3] == 222 and _oc(oracle, runs[1:], True) == []


def test_seqno_is_unsigned_64_bit(oracle):
    k = small_key(1)
    runs = [[brute.pack_entry(k, (1 << 63) - 1, PUT, vptr=1)], [brute.pack_entry(k, (1 << 63) + 5, PUT, vptr=2)]]
    assert brute.unpack(_oc(oracle, runs, False)[0])[3] == 2


# ---------------------------------------------------------------- special cases
def _distinct_keys(rs, n):
    keys = set()
    while len(keys) < n:
        keys.add(bytes(rs.randint(0, 256, size=32).astype(np.uint8)))
    return sorted(keys)


def test_two_runs_without_duplicates_is_a_plain_merge(oracle):
    rs = np.random.RandomState(3)
    keys = _distinct_keys(rs, 500)
    side = rs.rand(500) < 0.4
    a = [brute.pack_entry(k, i, PUT, vptr=i) for i, k in enumerate(keys) if side[i]]
    b = [brute.pack_entry(k, i, PUT, vptr=i) for i, k in enumerate(keys) if not side[i]]
    assert _oc(oracle, [a, b], False) == list(heapq.merge(a, b, key=lambda r: r[:32]))
    assert _oc(oracle, [a, b], True) == list(heapq.merge(a, b, key=lambda r: r[:32]))


def test_single_run_is_identity_or_tombstone_filter(oracle):
    rs = np.random.RandomState(4)
    keys = _distinct_keys(rs, 300)
    run = [brute.pack_entry(k, int(rs.randint(1 << 30)), TOMBSTONE if rs.rand() < 0.3 else PUT) for k in keys]
    assert _oc(oracle, [run], False) == run
    assert _oc(oracle, [run], True) == [r for r in run if brute.unpack(r)[2] == PUT]


def test_identical_key_sets_newest_run_wins_whole(oracle):
    rs = np.random.RandomState(5)
    keys = _distinct_keys(rs, 100)
    seq_base = [300, 900, 100, 500]  # run 1 is newest by seqno although run 0 is first
    runs = [[brute.pack_entry(k, base + i, PUT, vptr=base) for i, k in enumerate(keys)] for base in seq_base]
    assert _oc(oracle, runs, True) == runs[1]


def test_disjoint_ranges_concatenate(oracle):
    rs = np.random.RandomState(6)
    keys = _distinct_keys(rs, 300)
    parts = [keys[200:], keys[:80], keys[80:200]]
    runs = [[brute.pack_entry(k, j, PUT) for j, k in enumerate(p)] for p in parts]
    assert _oc(oracle, runs, False) == runs[1] + runs[2] + runs[0]


def test_all_tombstones_bottommost_is_empty_and_empty_runs_are_legal(oracle):
    rs = np.random.RandomState(7)
    keys = _distinct_keys(rs, 50)
    tomb = [brute.pack_entry(k, i, TOMBSTONE) for i, k in enumerate(keys)]
    assert _oc(oracle, [tomb, tomb[:10]], True) == []
    assert _oc(oracle, [[], tomb, []], False) == tomb
    assert _oc(oracle, [[], []], False) == [] and _oc(oracle, [], True) == []


def test_compaction_is_associative_when_inner_keeps_tombstones(oracle):
    rs = np.random.RandomState(8)
    for _ in range(60):
        a, b, c = brute.random_runs(rs, 3, 30, 50, (30, 31), tomb_p=0.3)
        # seqnos must make newer runs newer for nesting to be meaningful: any order works for the
        # definition (max seqno wins), so nesting is valid for arbitrary seqnos as long as ties
        # cannot occur across runs
        a = [r[:32] + (int.from_bytes(r[32:40], "little") * 4 + 0).to_bytes(8, "little") + r[40:] for r in a]
        b = [r[:32] + (int.from_bytes(r[32:40], "little") * 4 + 1).to_bytes(8, "little") + r[40:] for r in b]
        c = [r[:32] + (int.from_bytes(r[32:40], "little") * 4 + 2).to_bytes(8, "little") + r[40:] for r in c]
        for bottom in (False, True):
            inner = _oc(oracle, [a, b], False)
            assert _oc(oracle, [inner, c], bottom) == _oc(oracle, [a, b, c], bottom)


# ---------------------------------------------------------------- invariants on generated workloads
def check_compaction_invariants(runs_np, out_np, bottommost):
    """Properties that hold at any size (also used by the GPU parity tests)."""
    key_v = np.dtype((np.void, 32))
    out_keys = np.ascontiguousarray(out_np[:, :32]).view(key_v).ravel()
    # strictly ascending (np.void compares as bytes) => sorted and unique
    if out_keys.size > 1:
        ok = [bytes(out_keys[i]) < bytes(out_keys[i + 1]) for i in range(0, out_keys.size - 1, max(1, out_keys.size // 5000))]
        assert all(ok)
    newest = {}
    for r, run in enumerate(runs_np):
        seq = run[:, 32:40].copy().view("<u8").ravel()
        for i in range(run.shape[0]):
            k = run[i, :32].tobytes()
            cur = newest.get(k)
            if cur is None or seq[i] > cur[0]:
                newest[k] = (int(seq[i]), r, i)
    expect = []
    for k in sorted(newest):
        _, r, i = newest[k]
        if bottommost and runs_np[r][i, 40] == TOMBSTONE:
            continue
        expect.append(runs_np[r][i])
    assert out_np.shape[0] == len(expect)  # survivor count = deduplicated union minus dropped tombstones
    assert np.array_equal(out_np, np.stack(expect) if expect else np.zeros((0, 64), np.uint8))


def test_invariants_on_config1(oracle):
    from workloads import lsm
    w = lsm.config1()
    runs = [oracle.as_run(r) for r in w.runs]
    for bottom in (False, True):
        out = oracle.compact(runs, oracle.FLAG_BOTTOMMOST if bottom else 0)
        check_compaction_invariants(runs, out, bottom)
        if bottom:
            assert not (out[:, 40] == TOMBSTONE).any()


def test_invariants_on_scaled_config3(oracle):
    from workloads import lsm
    w = lsm.config3(scale=512)
    runs = [oracle.as_run(r) for r in w.runs]
    out = oracle.compact(runs, oracle.FLAG_BOTTOMMOST)
    check_compaction_invariants(runs, out, True)
    n_in = sum(r.shape[0] for r in runs)
    assert 0.60 < out.shape[0] / n_in < 0.76  # about 0.95 / 1.4 of the inputs survive


def test_planted_mistakes_are_caught(oracle):
    """The brute-force definition must disagree with plausible wrong merges (sanity of the pin)."""
    k = small_key(9)
    runs = [[brute.pack_entry(k, 5, PUT, vptr=1)], [brute.pack_entry(k, 9, TOMBSTONE, vptr=2)]]
    # a merge that prefers the lowest run index instead of the largest seqno would keep vptr=1
    assert brute.unpack(_oc(oracle, runs, False)[0])[3] == 2
    assert _oc(oracle, runs, True) == []


# ------------------------------------------------------------------ pointer rewrite (section 3.4)
def test_pointer_rewrite_against_plain_arithmetic(oracle):
    """remap_pointers on packed entries vs the rule written out with Python integers: PUTs inside the table
    move, tombstones and files outside the table do not; the identity table changes nothing."""
    rs = np.random.RandomState(3)
    raws = []
    for i in range(300):
        key = bytes(rs.randint(0, 256, size=32).astype(np.uint8))
        file_id, offset = int(rs.randint(0, 12)), int(rs.randint(0, 1 << 31))
        typ = brute.TOMBSTONE if i % 7 == 0 else brute.PUT
        raws.append(brute.pack_entry(key, i, typ, (file_id << 32) | offset if typ == brute.PUT else 0, 77, b"\x05" * 7, 9))
    run = brute.run_from_raw(sorted(raws, key=lambda r: r[:32]))
    n_files = 8  # files 8..11 are outside the table
    # files 0..7 concatenated into new file 100: base = start of each old file in the new one
    sizes = [int(rs.randint(1 << 31, 1 << 32)) for _ in range(n_files)]
    starts = [sum(sizes[:f]) for f in range(n_files)]  # may exceed 32 bits: the carry goes into the file field
    base = [((100 << 32) + st) for st in starts]
    got = oracle.remap_pointers(run, base)
    for before, after in zip(brute.raws_of(run), brute.raws_of(got)):
        key, seqno, typ, vptr, vlen = brute.unpack(before)
        key2, seqno2, typ2, vptr2, vlen2 = brute.unpack(after)
        assert (key, seqno, typ, vlen) == (key2, seqno2, typ2, vlen2) and before[41:48] == after[41:48] and before[60:] == after[60:]
        f, off = vptr >> 32, vptr & 0xFFFFFFFF
        assert vptr2 == ((100 << 32) + starts[f] + off if typ == brute.PUT and f < n_files else vptr)
    assert np.array_equal(oracle.remap_pointers(run, [f << 32 for f in range(12)]), run)
    assert np.array_equal(oracle.remap_pointers(run, []), run)


# ------------------------------------------------------------------ write-buffer flush (section 2.2)
def test_flush_buffer_equals_merging_one_entry_runs(oracle):
    """Flushing a buffer = compacting its entries as one-entry runs, the last written first (so that equal seqnos go
    to the later write): checked against the sort-and-deduplicate reference on raw bytes."""
    rs = np.random.RandomState(21)
    alphabet = [bytes(rs.randint(0, 256, size=32).astype(np.uint8)) for _ in range(60)]
    for n in (0, 1, 2, 257, 700):
        raws = [brute.pack_entry(alphabet[int(rs.randint(len(alphabet)))], int(rs.randint(0, 5)) if i % 3 else int(rs.randint(0, 1 << 40)),
                                 TOMBSTONE if rs.rand() < 0.3 else PUT, i, i % 7) for i in range(n)]
        want = brute.compact([[r] for r in reversed(raws)], False)
        got = oracle.flush_buffer(brute.run_from_raw(raws))
        assert brute.raws_of(got) == want
        keys = [r[:32] for r in brute.raws_of(got)]
        assert keys == sorted(set(r[:32] for r in raws))
