"""ctypes front end of the C checker in this directory (test infrastructure only).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this module.
Arrays are numpy: a run is a C-contiguous uint8 array of shape [n, 64].
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Sequence, Tuple

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "lsm_oracle.c")
_LIB = os.path.join(_DIR, "liblsm_oracle.so")

FLAG_BOTTOMMOST = 1
ENTRY_BYTES = 64

HIT_DTYPE = np.dtype([("vptr", "<u8"), ("vlen", "<u4"), ("run_idx", "<u4")])
ENTRY_DTYPE = np.dtype([("key", "u1", (32,)), ("seqno", "<u8"), ("type", "u1"), ("pad0", "u1", (7,)),
                        ("vptr", "<u8"), ("vlen", "<u4"), ("pad1", "<u4")])
assert ENTRY_DTYPE.itemsize == 64 and HIT_DTYPE.itemsize == 16


def build(force: bool = False) -> str:
    """Compile the checker with gcc (a second or so)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        L.oracle_key_cmp.restype = C.c_int
        L.oracle_key_cmp.argtypes = [C.c_void_p, C.c_void_p]
        L.oracle_compact.restype = C.c_uint64
        L.oracle_compact.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p]
        L.oracle_probe.restype = None
        L.oracle_probe.argtypes = [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32, C.c_void_p, C.c_void_p,
                                   C.c_uint32, C.c_void_p, C.c_void_p]
        L.oracle_build_fences.restype = None
        L.oracle_build_fences.argtypes = [C.c_void_p, C.c_uint64, C.c_uint32, C.c_void_p]
        L.oracle_bloom_blocks.restype = C.c_uint64
        L.oracle_bloom_blocks.argtypes = [C.c_uint64, C.c_uint32]
        L.oracle_build_bloom.restype = None
        L.oracle_build_bloom.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.oracle_bloom_may_contain.restype = C.c_int
        L.oracle_bloom_may_contain.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.oracle_key_hashes.restype = None
        L.oracle_key_hashes.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p]
        L.oracle_hash_index_buckets.restype = C.c_uint64
        L.oracle_hash_index_buckets.argtypes = [C.c_uint64]
        L.oracle_hash_index_check.restype = C.c_int
        L.oracle_hash_index_check.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64]
        L.oracle_levels.restype = C.c_uint32
        L.oracle_levels.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32]
        L.oracle_cost.restype = C.c_double
        L.oracle_cost.argtypes = [C.c_double] * 4 + [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32] + [C.c_double] * 3
        L.oracle_policy_choose.restype = None
        L.oracle_policy_choose.argtypes = ([C.c_double] * 4 + [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
                                           + [C.c_double] * 3 + [C.c_void_p, C.c_void_p])
        _lib = L
    return _lib


def as_run(a) -> np.ndarray:
    """Anything holding n x 64 bytes (numpy, or a CPU torch tensor [n, 8] int64) -> uint8 [n, 64]."""
    if hasattr(a, "detach"):
        a = a.detach().cpu().contiguous().numpy()
    a = np.ascontiguousarray(a)
    return a.view(np.uint8).reshape(-1, ENTRY_BYTES)


def _run_table(runs: Sequence[np.ndarray]):
    ptrs = (C.c_void_p * max(1, len(runs)))(*[r.ctypes.data for r in runs])
    lens = (C.c_uint64 * max(1, len(runs)))(*[r.shape[0] for r in runs])
    return ptrs, lens


def key_cmp(a: bytes, b: bytes) -> int:
    assert len(a) == 32 and len(b) == 32
    return int(lib().oracle_key_cmp(C.c_char_p(a), C.c_char_p(b)))


def compact(runs: Sequence, flags: int = 0) -> np.ndarray:
    """Merge sorted runs (runs[0] newest).  Returns the surviving entries, uint8 [n_out, 64]."""
    runs = [as_run(r) for r in runs]
    total = sum(r.shape[0] for r in runs)
    out = np.zeros((max(total, 1), ENTRY_BYTES), dtype=np.uint8)
    ptrs, lens = _run_table(runs)
    n_out = lib().oracle_compact(ptrs, lens, len(runs), flags, out.ctypes.data)
    return out[:n_out]


def probe(qkeys, n_blocks, runs: Sequence) -> Tuple[np.ndarray, np.ndarray]:
    """qkeys: uint8 [n_req, max_blocks, 32] (or anything with that memory image), n_blocks:
    uint32 [n_req]; runs newest first.  Returns (hit_len uint32 [n_req], hits HIT_DTYPE
    [n_req, max_blocks])."""
    if hasattr(qkeys, "detach"):
        qkeys = qkeys.detach().cpu().contiguous().numpy()
    if hasattr(n_blocks, "detach"):
        n_blocks = n_blocks.detach().cpu().numpy()
    n_req = int(np.asarray(n_blocks).shape[0])
    q = np.ascontiguousarray(qkeys).view(np.uint8).reshape(n_req, -1, 32) if n_req else np.zeros((0, 1, 32), np.uint8)
    max_blocks = q.shape[1]
    nb = np.ascontiguousarray(n_blocks, dtype=np.uint32)
    assert (nb <= max_blocks).all()
    runs = [as_run(r) for r in runs]
    ptrs, lens = _run_table(runs)
    hit_len = np.zeros(max(n_req, 1), dtype=np.uint32)
    hits = np.zeros((max(n_req, 1), max_blocks), dtype=HIT_DTYPE)
    lib().oracle_probe(q.ctypes.data, nb.ctypes.data, n_req, max_blocks, ptrs, lens, len(runs),
                       hit_len.ctypes.data, hits.ctypes.data)
    return hit_len[:n_req], hits[:n_req]


def build_fences(run, stride: int) -> np.ndarray:
    run = as_run(run)
    n = run.shape[0]
    out = np.zeros(((n + stride - 1) // stride, 32), dtype=np.uint8)
    lib().oracle_build_fences(run.ctypes.data, n, stride, out.ctypes.data)
    return out


def flush_buffer(buffer) -> np.ndarray:
    """The write buffer as a sorted run (section 2.2): ascending by key, of several versions of a key the one with
    the largest seqno, among equal seqnos the one written last (= later in the buffer)."""
    buf = as_run(buffer)
    rec = buf.view(ENTRY_DTYPE).reshape(-1)
    order = sorted(range(buf.shape[0]), key=lambda i: (bytes(rec["key"][i]), -int(rec["seqno"][i]), -i))
    keep, last = [], None
    for i in order:
        k = bytes(rec["key"][i])
        if k != last:
            keep.append(i)
            last = k
    return buf[keep] if keep else buf[:0]


def remap_pointers(run, base) -> np.ndarray:
    """Pointer rewrite for merged tensor files (section 3.4): a value pointer is (file_id << 32) | offset;
    every PUT whose file_id is inside the table gets base[file_id] + offset, everything else stays."""
    out = as_run(run).copy()
    rec = out.view(ENTRY_DTYPE).reshape(-1)
    base = np.asarray(base, dtype=np.uint64)
    for i in range(rec.shape[0]):
        file_id, offset = int(rec["vptr"][i]) >> 32, int(rec["vptr"][i]) & 0xFFFFFFFF
        if int(rec["type"][i]) == 0 and file_id < base.shape[0]:
            rec["vptr"][i] = (int(base[file_id]) + offset) & 0xFFFFFFFFFFFFFFFF
    return out


def key_hashes(run) -> np.ndarray:
    """The filter hash h of every key of a run (uint64 [n]); see the C source."""
    run = as_run(run)
    out = np.zeros(run.shape[0], dtype=np.uint64)
    lib().oracle_key_hashes(run.ctypes.data, run.shape[0], out.ctypes.data)
    return out


def hash_index_buckets(n: int) -> int:
    return int(lib().oracle_hash_index_buckets(n))


def hash_index_check(run, table) -> int:
    """0 if `table` (bytes, n_buckets x 64) is a valid hash index of the run, else the number of the broken rule."""
    run = as_run(run)
    table = np.ascontiguousarray(table).view(np.uint8).reshape(-1, 64)
    return int(lib().oracle_hash_index_check(run.ctypes.data, run.shape[0], table.ctypes.data, table.shape[0]))


def bloom_blocks(n: int, bits_per_key: int) -> int:
    return int(lib().oracle_bloom_blocks(n, bits_per_key))


def build_bloom(run, n_blocks: int) -> np.ndarray:
    """Filter bytes [n_blocks, 16] (section 2.2, Bloom filters; format in the C source)."""
    run = as_run(run)
    out = np.zeros((n_blocks, 16), dtype=np.uint8)
    lib().oracle_build_bloom(run.ctypes.data, run.shape[0], out.ctypes.data, n_blocks)
    return out


def bloom_may_contain(filt: np.ndarray, key: bytes) -> bool:
    filt = np.ascontiguousarray(filt, dtype=np.uint8)
    kb = (C.c_uint8 * 32).from_buffer_copy(key)
    return bool(lib().oracle_bloom_may_contain(filt.ctypes.data, filt.shape[0], kb))


def levels(n_entries: int, buffer_entries: int, T: int) -> int:
    return int(lib().oracle_levels(n_entries, buffer_entries, T))


def cost(w, s, r, z, n_entries, buffer_entries, T, K, B, p, d) -> float:
    return float(lib().oracle_cost(w, s, r, z, n_entries, buffer_entries, T, K, B, p, d))


def policy_choose(w, s, r, z, n_entries, buffer_entries, t_min, t_max, B, p, d) -> Tuple[int, int]:
    bt, bk = C.c_uint32(0), C.c_uint32(0)
    lib().oracle_policy_choose(w, s, r, z, n_entries, buffer_entries, t_min, t_max, B, p, d,
                               C.byref(bt), C.byref(bk))
    return int(bt.value), int(bk.value)
