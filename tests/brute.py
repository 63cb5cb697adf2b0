"""Plain-Python definitions used to pin the C checker on tiny inputs.

Deliberately a different language and a different method from oracle/lsm_oracle.c:
compaction is "concatenate, sort, keep the first of each key group, filter"; lookup is an
exhaustive scan of every entry of every run.  Entries are tuples
(key: bytes[32], seqno: int, type: int, raw: bytes[64]).
"""
from __future__ import annotations

import struct
from typing import List, Sequence, Tuple

import numpy as np

PUT, TOMBSTONE = 0, 1


def pack_entry(key: bytes, seqno: int, typ: int, vptr: int = 0, vlen: int = 0, pad0: bytes = b"\0" * 7,
               pad1: int = 0) -> bytes:
    assert len(key) == 32 and len(pad0) == 7
    return key + struct.pack("<QB7sQII", seqno, typ, pad0, vptr, vlen, pad1)


def unpack(raw: bytes):
    seqno, typ, _pad0, vptr, vlen, _pad1 = struct.unpack("<QB7sQII", raw[32:])
    return raw[:32], seqno, typ, vptr, vlen


def run_from_raw(raws: Sequence[bytes]) -> np.ndarray:
    a = np.frombuffer(b"".join(raws), dtype=np.uint8).reshape(-1, 64) if raws else np.zeros((0, 64), np.uint8)
    return a.copy()


def raws_of(run: np.ndarray) -> List[bytes]:
    run = np.ascontiguousarray(run).view(np.uint8).reshape(-1, 64)
    return [run[i].tobytes() for i in range(run.shape[0])]


def compact(runs: Sequence[Sequence[bytes]], bottommost: bool) -> List[bytes]:
    """runs[r] = list of 64-byte entries (run 0 newest).  Sort + dedup definition."""
    allv = []
    for r, run in enumerate(runs):
        for raw in run:
            key, seqno, typ, _, _ = unpack(raw)
            allv.append((key, -seqno, r, typ, raw))
    allv.sort(key=lambda t: (t[0], t[1], t[2]))
    out, last = [], None
    for key, _, _, typ, raw in allv:
        if key == last:
            continue
        last = key
        if bottommost and typ == TOMBSTONE:
            continue
        out.append(raw)
    return out


def newest(runs: Sequence[Sequence[bytes]], key: bytes):
    """Exhaustive scan: (seqno, run, raw) of the newest version of key, or None."""
    best = None
    for r, run in enumerate(runs):
        for raw in run:
            if raw[:32] == key:
                seqno = struct.unpack("<Q", raw[32:40])[0]
                if best is None or seqno > best[0]:
                    best = (seqno, r, raw)
    return best


def probe(runs: Sequence[Sequence[bytes]], requests: Sequence[Sequence[bytes]], max_blocks: int
          ) -> Tuple[List[int], List[List[Tuple[int, int, int]]]]:
    hit_len, hits = [], []
    for req in requests:
        row = [(0, 0, 0)] * max_blocks
        j = 0
        for j, key in enumerate(req):
            b = newest(runs, key)
            if b is None or unpack(b[2])[2] != PUT:
                break
            _, _, _, vptr, vlen = unpack(b[2])
            row[j] = (vptr, vlen, b[1])
        else:
            j = len(req)
        hit_len.append(j)
        hits.append(row)
    return hit_len, hits


def random_runs(rs: np.random.RandomState, n_runs: int, max_len: int, alphabet: int, vary_bytes: Sequence[int],
                tomb_p: float = 0.3, seq_space: int = 1 << 20, force_seq_ties: bool = False) -> List[List[bytes]]:
    """Tiny runs over a small key alphabet so duplicates, ties and tombstones all occur.
    Keys differ only in the byte positions `vary_bytes`."""
    def mk_key(code: int) -> bytes:
        # byte i of the code goes to position vary_bytes[i]; distinct codes -> distinct keys
        k = bytearray(32)
        for i, pos in enumerate(vary_bytes):
            k[pos] = (code >> (8 * i)) & 0xFF
        return bytes(k)

    assert alphabet <= 256 ** len(vary_bytes)
    runs = []
    for _ in range(n_runs):
        n = int(rs.randint(0, max_len + 1))
        codes = sorted(set(int(c) for c in rs.randint(0, alphabet, size=n)))
        keys = sorted(set(mk_key(c) for c in codes))
        run = []
        for key in keys:
            seqno = int(rs.randint(0, 4)) if force_seq_ties else int(rs.randint(0, seq_space))
            typ = TOMBSTONE if rs.rand() < tomb_p else PUT
            pad0 = bytes(rs.randint(0, 256, size=7).astype(np.uint8))
            run.append(pack_entry(key, seqno, typ, int(rs.randint(0, 1 << 62)), int(rs.randint(0, 1 << 31)), pad0,
                                  int(rs.randint(0, 1 << 31))))
        runs.append(run)
    return runs


def tie_group_runs(rs: np.random.RandomState, n_runs: int, n_heads: int, long_groups: int = 0) -> List[List[bytes]]:
    """Runs whose keys fall into groups that share their first 14 bytes and differ somewhere in
    bytes 14..31 (each of the later byte ranges decides for some pair).  Most groups have one to
    eight members; `long_groups` of them have forty.  Every key is in a random subset of the runs
    with random seqnos, so groups interleave runs and versions."""
    heads = sorted(set(bytes(rs.randint(0, 256, size=14).astype(np.uint8)) for _ in range(n_heads)))
    spots = [14, 15, 16, 20, 23, 24, 31]  # byte that tells two tails of a group apart
    runs: List[List[bytes]] = [[] for _ in range(n_runs)]
    for h, head in enumerate(heads):
        size = 40 if h < long_groups else int(rs.choice([1, 1, 1, 2, 3, 5, 8]))
        tails = set()
        while len(tails) < size:
            t = bytearray(18)
            for _ in range(int(rs.randint(1, 3))):
                t[spots[int(rs.randint(len(spots)))] - 14] = int(rs.randint(0, 4))
            tails.add(bytes(t))
        for tail in tails:
            for j in range(n_runs):
                if rs.rand() < 0.5:
                    typ = TOMBSTONE if rs.rand() < 0.2 else PUT
                    runs[j].append(pack_entry(head + tail, int(rs.randint(0, 1 << 40)), typ, int(rs.randint(0, 1 << 62)),
                                              j, bytes([j] * 7), h & 0x7FFFFFFF))
    return [sorted(r, key=lambda raw: raw[:32]) for r in runs]


def close_first_words_runs(rs: np.random.RandomState, n_runs: int, per_run: int, separate: bool) -> List[List[bytes]]:
    """Keys whose first 8 bytes take three values: two that differ only in their last bit and one far away, so
    that any fixed-width scaling of the first word maps the close pair to one value.  With `separate` the two
    close values never occur in the same run (run j holds only one of them), otherwise every run mixes them."""
    a = bytes([0x10] + [0] * 7)
    b = bytes([0x10] + [0] * 6 + [1])
    far = bytes([0xF0] + [0] * 7)
    runs = []
    for j in range(n_runs):
        firsts = [a if j % 2 == 0 else b, far] if separate else [a, b, far]
        keys = set()
        while len(keys) < per_run:
            keys.add(firsts[int(rs.randint(len(firsts)))] + bytes(rs.randint(0, 256, size=3).astype(np.uint8)) + bytes(21))
        run = [pack_entry(key, int(rs.randint(0, 1 << 40)), TOMBSTONE if rs.rand() < 0.2 else PUT, int(rs.randint(0, 1 << 62)), j,
                          bytes([j] * 7), j) for key in sorted(keys)]
        runs.append(run)
    return runs
