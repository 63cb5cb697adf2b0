"""The checker's side of the hash index: the key hash against the published definition worked out with Python
integers, and the validity check against tables built here, slot by slot, from the format's statement (in
include/lsm_index.h, at lsm_hash_index_t) - one valid table per case and one planted mistake per rule."""
import numpy as np
import pytest

import brute

M64 = (1 << 64) - 1
NONE = 0xFFFFFFFF


def _mix(x):
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & M64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & M64
    x ^= x >> 31
    return x


def _hash(key: bytes) -> int:
    h = 0x5EED251116138
    for i in range(4):
        h = _mix(h ^ int.from_bytes(key[8 * i:8 * i + 8], "big"))
    return h


def _run(rs, n):
    keys = sorted({bytes(rs.randint(0, 256, 32, dtype=np.uint8)) for _ in range(n)})
    return keys, brute.run_from_raw([brute.pack_entry(k, 1 + i, 0) for i, k in enumerate(keys)])


def _table(keys, order=None):
    """A valid table by the format's statement; `order` permutes the keys first (which eight a crowded bucket keeps).
    Returns the table as [n_buckets, 64] bytes and, per bucket, the (tag, position) pairs of all its keys."""
    n = len(keys)
    n_buckets = max(1, -(-n // 4))
    members = [[] for _ in range(n_buckets)]
    for pos in (int(p) for p in (order if order is not None else range(n))):
        h = _hash(keys[pos])
        members[((h >> 32) * n_buckets) >> 32].append((h & 0x7FFF, pos))
    table = np.zeros((n_buckets, 64), dtype=np.uint8)
    for b, m in enumerate(members):
        tags = [t for t, _ in m[:8]] + [0] * (8 - min(8, len(m)))
        poss = [p for _, p in m[:8]] + [NONE] * (8 - min(8, len(m)))
        if len(m) > 8:
            tags[0] |= 0x8000
        table[b, :16] = np.array(tags, dtype="<u2").view(np.uint8)
        table[b, 16:48] = np.array(poss, dtype="<u4").view(np.uint8)
    return table, members


def _set_tag(t, b, k, v):
    t[b, 2 * k:2 * k + 2] = np.array([v], dtype="<u2").view(np.uint8)


def _set_pos(t, b, k, v):
    t[b, 16 + 4 * k:20 + 4 * k] = np.array([v], dtype="<u4").view(np.uint8)


def test_key_hash_follows_the_definition(oracle):
    rs = np.random.RandomState(3)
    keys, run = _run(rs, 300)
    got = oracle.key_hashes(run)
    assert got.dtype == np.uint64 and got.tolist() == [_hash(k) for k in keys]
    assert oracle.key_hashes(run[:0]).shape == (0,)
    assert [oracle.hash_index_buckets(n) for n in (0, 1, 4, 5, 4096, 4097)] == [1, 1, 1, 2, 1024, 1025]


@pytest.mark.parametrize("n", [0, 1, 9, 40, 3000])
def test_valid_tables_pass(oracle, n):
    rs = np.random.RandomState(n)
    keys, run = _run(rs, n)
    slots, members = _table(keys)
    assert oracle.hash_index_check(run, slots) == 0
    # the slots of a bucket in another order, and other keys kept in the crowded buckets: still valid
    slots2, _ = _table(keys, order=list(rs.permutation(len(keys))))
    assert oracle.hash_index_check(run, slots2) == 0
    if n == 3000:
        assert any(len(m) > 8 for m in members) and any(len(m) == 8 for m in members)   # both cases occur


def test_every_rule_is_enforced(oracle):
    rs = np.random.RandomState(11)
    keys, run = _run(rs, 3000)
    good, members = _table(keys)
    full = next(b for b, m in enumerate(members) if len(m) == 8)
    crowded = next(b for b, m in enumerate(members) if len(m) > 8)
    some = next(b for b, m in enumerate(members) if 1 <= len(m) <= 6)
    other = next(b for b, m in enumerate(members) if 1 <= len(m) <= 6 and b != some)

    def broken(*edits):
        t = good.copy()
        for f, b, k, v in edits:
            f(t, b, k, v)
        return oracle.hash_index_check(run, t)

    assert oracle.hash_index_check(run, good[:-1]) == 1                                              # bucket count
    assert broken((_set_pos, some, 0, 3000)) == 2                                                    # position outside the run
    assert broken((_set_tag, some, 0, members[some][0][0] ^ 0x10)) == 3                              # wrong tag
    assert broken((_set_tag, some, 7, members[other][0][0]), (_set_pos, some, 7, members[other][0][1])) == 3   # key in a foreign bucket
    assert broken((_set_tag, some, 7, members[some][0][0]), (_set_pos, some, 7, members[some][0][1])) == 4     # listed twice
    assert broken((_set_tag, some, 0, members[some][0][0] | 0x8000)) == 5                            # crowded bit without need
    assert broken((_set_tag, some, 0, 0), (_set_pos, some, 0, NONE)) == 6                            # a key dropped
    assert broken((_set_tag, full, 0, members[full][0][0] | 0x8000)) == 5                            # eight keys fit: no bit
    assert broken((_set_tag, crowded, 0, members[crowded][0][0])) == 7                               # crowded without the bit
    assert broken((_set_tag, crowded, 6, 0), (_set_pos, crowded, 6, NONE)) == 7                      # crowded holding seven
    assert broken((_set_tag, some, 3, members[some][3][0] | 0x8000 if len(members[some]) > 3 else 0x8000)) == 8   # bit 15 in another field
    assert broken((_set_tag, some, 7, 5)) == 9                                                       # a tag on an empty slot
    t = good.copy()
    t[some, 50] = 1
    assert oracle.hash_index_check(run, t) == 10                                                     # the rest of a bucket is zero
