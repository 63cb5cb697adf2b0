"""ctypes binding of liblsm_index.so (same names as the C entry points, marshalling only).

Tensors are torch tensors on the GPU:
  run       int64 [n, 8]   (64-byte entries; see include/lsm_index.h for the field layout)
  fences    int64 [n_f, 4] (32-byte keys)
  queries   int64 [n_req, max_blocks, 4] keys + int32 [n_req] block counts
  hits      int64 [n_req, max_blocks, 2] (vptr | vlen + run_idx << 32), int32 [n_req] hit_len
The library must have been built (python -c "import __graft_entry__ as g; g.build()");
there is no fallback: a missing library raises at the first call.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

import torch

LSM_BOTTOMMOST = 1
LSM_VALIDATE = 2
LSM_MAX_RUNS = 64
LSM_MAX_BLOCKS = 256

_HERE = os.path.dirname(os.path.abspath(__file__))


def library_path() -> str:
    return os.path.join(_HERE, "liblsm_index.so")


class LsmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {lsm_strerror(code)} ({code})")


class _Run(C.Structure):
    _fields_ = [("entries", C.c_void_p), ("n", C.c_uint64)]


class _Out(C.Structure):
    _fields_ = [("entries", C.c_void_p), ("capacity", C.c_uint64), ("n_out", C.c_void_p), ("fence_keys", C.c_void_p),
                ("fence_stride", C.c_uint32), ("key_hashes", C.c_void_p)]


class _Fence(C.Structure):
    _fields_ = [("keys", C.c_void_p), ("n", C.c_uint64), ("stride", C.c_uint32)]


class _Bloom(C.Structure):
    _fields_ = [("blocks", C.c_void_p), ("n_blocks", C.c_uint64)]


class _HashIndex(C.Structure):
    _fields_ = [("buckets", C.c_void_p), ("n_buckets", C.c_uint64)]


class _TreeRun(C.Structure):
    _fields_ = [("run", _Run), ("fence", _Fence), ("bloom", _Bloom), ("level", C.c_uint32), ("index", _HashIndex)]


class _Tree(C.Structure):
    _fields_ = [("runs", C.POINTER(_TreeRun)), ("n_runs", C.c_uint32)]


class _Queries(C.Structure):
    _fields_ = [("keys", C.c_void_p), ("n_blocks", C.c_void_p), ("n_req", C.c_uint32), ("max_blocks", C.c_uint32)]


class _Hits(C.Structure):
    _fields_ = [("hit_len", C.c_void_p), ("hits", C.c_void_p)]


class _CompactEvents(C.Structure):
    _fields_ = [("before_partition", C.c_void_p), ("before_merge", C.c_void_p), ("after_merge", C.c_void_p)]


class _Remap(C.Structure):
    _fields_ = [("base", C.c_void_p), ("n_files", C.c_uint32)]


class _Ranges(C.Structure):
    _fields_ = [("lo_keys", C.c_void_p), ("hi_keys", C.c_void_p), ("n_ranges", C.c_uint32), ("max_entries", C.c_uint32)]


class _RangeOut(C.Structure):
    _fields_ = [("entries", C.c_void_p), ("counts", C.c_void_p)]


class _CompactJob(C.Structure):
    _fields_ = [("runs", C.POINTER(_Run)), ("n_runs", C.c_uint32), ("flags", C.c_uint32), ("out", _Out)]


class _PolicyInput(C.Structure):
    _fields_ = [("w", C.c_double), ("s", C.c_double), ("r", C.c_double), ("z", C.c_double), ("n_entries", C.c_uint64),
                ("buffer_entries", C.c_uint64), ("B", C.c_double), ("p", C.c_double), ("d", C.c_double)]


class _DriverEvent(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("level", C.c_uint32), ("a", C.c_uint32), ("b", C.c_uint32), ("n_in", C.c_uint64),
                ("n_out", C.c_uint64), ("mix", C.c_double * 4), ("d", C.c_double)]


_DriverObserver = C.CFUNCTYPE(None, C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64)


class _DriverConfig(C.Structure):
    _fields_ = [("buffer_entries", C.c_uint64), ("size_ratio", C.c_uint32), ("runs_per_level", C.c_uint32),
                ("window_ops", C.c_uint64), ("shift_threshold", C.c_double), ("t_min", C.c_uint32), ("t_max", C.c_uint32),
                ("page_entries", C.c_double), ("filter_fpr", C.c_double), ("fence_stride", C.c_uint32), ("bloom_bits", C.c_uint32),
                ("hash_index_from", C.c_uint64), ("observer", _DriverObserver), ("observer_ctx", C.c_void_p)]


_lib: Optional[C.CDLL] = None


def _load(path: Optional[str] = None) -> C.CDLL:
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it first (__graft_entry__.build()); there is no CPU fallback")
    L = C.CDLL(path)
    L.lsm_compact.restype = C.c_int
    L.lsm_compact.argtypes = [C.POINTER(_Run), C.c_uint32, C.c_uint32, C.POINTER(_Out), C.c_void_p, C.c_size_t, C.c_void_p]
    L.lsm_compact_timed.restype = C.c_int
    L.lsm_compact_timed.argtypes = L.lsm_compact.argtypes + [C.POINTER(_CompactEvents)]
    L.lsm_compact_remap.restype = C.c_int
    L.lsm_compact_remap.argtypes = L.lsm_compact.argtypes + [C.POINTER(_Remap), C.POINTER(_CompactEvents)]
    L.lsm_compact_static.restype = C.c_int
    L.lsm_compact_static.argtypes = [C.POINTER(_Run), C.c_uint32, C.c_uint32, C.POINTER(_Out), C.c_void_p]
    L.lsm_compact_workspace_bytes.restype = C.c_size_t
    L.lsm_compact_workspace_bytes.argtypes = [C.POINTER(C.c_uint64), C.c_uint32]
    L.lsm_build_fences.restype = C.c_int
    L.lsm_build_fences.argtypes = [C.POINTER(_Run), C.c_uint32, C.c_void_p, C.c_void_p]
    L.lsm_flush_workspace_bytes.restype = C.c_size_t
    L.lsm_flush_workspace_bytes.argtypes = [C.c_uint64]
    L.lsm_flush_buffer.restype = C.c_int
    L.lsm_flush_buffer.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(_Out), C.c_void_p, C.c_size_t, C.c_void_p]
    L.lsm_bloom_blocks.restype = C.c_uint64
    L.lsm_bloom_blocks.argtypes = [C.c_uint64, C.c_uint32]
    L.lsm_build_bloom.restype = C.c_int
    L.lsm_build_bloom.argtypes = [C.POINTER(_Run), C.c_void_p, C.c_uint64, C.c_void_p]
    L.lsm_build_bloom_batch.restype = C.c_int
    L.lsm_build_bloom_batch.argtypes = [C.POINTER(_Run), C.POINTER(C.c_void_p), C.POINTER(C.c_uint64), C.c_uint32, C.c_void_p]
    L.lsm_bloom_workspace_bytes.restype = C.c_size_t
    L.lsm_bloom_workspace_bytes.argtypes = [C.c_uint64, C.c_uint64]
    L.lsm_hash_keys.restype = C.c_int
    L.lsm_hash_keys.argtypes = [C.POINTER(_Run), C.c_void_p, C.c_void_p]
    L.lsm_build_bloom_hashed.restype = C.c_int
    L.lsm_build_bloom_hashed.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_uint64, C.c_void_p, C.c_size_t, C.c_void_p]
    L.lsm_hash_index_buckets.restype = C.c_uint64
    L.lsm_hash_index_buckets.argtypes = [C.c_uint64]
    L.lsm_hash_index_workspace_bytes.restype = C.c_size_t
    L.lsm_hash_index_workspace_bytes.argtypes = [C.c_uint64]
    L.lsm_build_hash_index.restype = C.c_int
    L.lsm_build_hash_index.argtypes = [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    L.lsm_probe.restype = C.c_int
    L.lsm_probe.argtypes = [C.POINTER(_Queries), C.POINTER(_Tree), C.POINTER(_Hits), C.c_void_p]
    L.lsm_probe_length.restype = C.c_int
    L.lsm_probe_length.argtypes = [C.POINTER(_Queries), C.POINTER(_Tree), C.c_void_p, C.c_void_p]
    L.lsm_range_bounds.restype = C.c_int
    L.lsm_range_bounds.argtypes = [C.POINTER(_Tree), C.c_char_p, C.c_char_p, C.c_void_p, C.c_void_p]
    L.lsm_range_scan.restype = C.c_int
    L.lsm_range_scan.argtypes = [C.POINTER(_Ranges), C.POINTER(_Tree), C.POINTER(_RangeOut), C.c_void_p]
    L.lsm_compact_batch_workspace_bytes.restype = C.c_size_t
    L.lsm_compact_batch_workspace_bytes.argtypes = [C.POINTER(_CompactJob), C.c_uint32]
    L.lsm_compact_batch.restype = C.c_int
    L.lsm_compact_batch.argtypes = [C.POINTER(_CompactJob), C.c_uint32, C.c_void_p, C.c_size_t, C.c_void_p]
    L.lsm_policy_levels.restype = C.c_uint32
    L.lsm_policy_levels.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32]
    L.lsm_policy_cost.restype = C.c_double
    L.lsm_policy_cost.argtypes = [C.POINTER(_PolicyInput), C.c_uint32, C.c_uint32]
    L.lsm_policy_choose.restype = C.c_int
    L.lsm_policy_choose.argtypes = [C.POINTER(_PolicyInput), C.c_uint32, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    L.lsm_policy_filter_fpr.restype = C.c_double
    L.lsm_policy_filter_fpr.argtypes = [C.c_uint32]
    L.lsm_driver_create.restype = C.c_int
    L.lsm_driver_create.argtypes = [C.POINTER(_DriverConfig), C.c_void_p, C.POINTER(C.c_void_p)]
    L.lsm_driver_destroy.restype = None
    L.lsm_driver_destroy.argtypes = [C.c_void_p]
    L.lsm_driver_load_run.restype = C.c_int
    L.lsm_driver_load_run.argtypes = [C.c_void_p, C.c_uint32, C.c_void_p, C.c_uint64]
    L.lsm_driver_note_writes.restype = C.c_int
    L.lsm_driver_note_writes.argtypes = [C.c_void_p, C.c_uint64]
    L.lsm_driver_note_reads.restype = C.c_int
    L.lsm_driver_note_reads.argtypes = [C.c_void_p, C.c_uint64, C.c_uint64, C.c_uint64]
    L.lsm_driver_flush.restype = C.c_int
    L.lsm_driver_flush.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
    L.lsm_driver_flush_unsorted.restype = C.c_int
    L.lsm_driver_flush_unsorted.argtypes = [C.c_void_p, C.c_void_p, C.c_uint64]
    L.lsm_driver_flush_many.restype = C.c_int
    L.lsm_driver_flush_many.argtypes = [C.POINTER(C.c_void_p), C.POINTER(C.c_void_p), C.POINTER(C.c_uint64), C.c_uint32]
    L.lsm_driver_probe.restype = C.c_int
    L.lsm_driver_probe.argtypes = [C.c_void_p, C.POINTER(_Queries), C.POINTER(_Hits)]
    L.lsm_driver_levels.restype = C.c_uint32
    L.lsm_driver_levels.argtypes = [C.c_void_p]
    L.lsm_driver_level.restype = C.c_int
    L.lsm_driver_level.argtypes = [C.c_void_p, C.c_uint32, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    L.lsm_driver_tree.restype = C.c_int
    L.lsm_driver_tree.argtypes = [C.c_void_p, C.POINTER(_TreeRun), C.c_uint32, C.POINTER(C.c_uint32)]
    L.lsm_driver_target.restype = C.c_int
    L.lsm_driver_target.argtypes = [C.c_void_p, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
    L.lsm_driver_log.restype = C.c_uint64
    L.lsm_driver_log.argtypes = [C.c_void_p, C.c_uint64, C.POINTER(_DriverEvent), C.c_uint64]
    L.lsm_driver_read.restype = C.c_int
    L.lsm_driver_read.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t]
    L.lsm_strerror.restype = C.c_char_p
    L.lsm_strerror.argtypes = [C.c_int]
    _lib = L
    return L


def _dev(t: torch.Tensor, what: str) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError(f"{what} must be a GPU tensor")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


def _count(t: torch.Tensor, what: str) -> torch.Tensor:
    """A tensor the kernels write a count to: device memory, or pinned host memory (which the GPU addresses
    directly, so that the host can read the count after a stream synchronisation, without a copy)."""
    if not (t.is_cuda or t.is_pinned()):
        raise ValueError(f"{what} must be a GPU tensor or pinned host memory")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    return t


_raw_current_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)


def _stream_ptr(stream) -> int:
    if stream is None:
        if _raw_current_stream is not None:   # the handle alone: building a Stream object costs more than a small launch
            return int(_raw_current_stream(torch.cuda.current_device()))
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) if hasattr(stream, "cuda_stream") else int(stream)


def lsm_strerror(code: int) -> str:
    return _load().lsm_strerror(code).decode()


def lsm_compact_workspace_bytes(run_lens: Sequence[int]) -> int:
    arr = (C.c_uint64 * max(1, len(run_lens)))(*run_lens)
    return int(_load().lsm_compact_workspace_bytes(arr, len(run_lens)))


def lsm_compact(runs: Sequence[torch.Tensor], flags: int = 0, out: Optional[torch.Tensor] = None,
                n_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None,
                events: Optional[Tuple[int, int, int]] = None, remap: Optional[torch.Tensor] = None,
                fences: Optional[torch.Tensor] = None, fence_stride: int = 64,
                key_hashes: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """Merge sorted runs (runs[0] newest).  Returns (out, n_out): out is int64 [capacity, 8]
    whose first n_out rows are the result, n_out a one-element int64 tensor on the device (or, if the caller passes one, in
    pinned host memory: the count can then be read after a stream synchronisation without a copy).
    `events` = three raw hipEvent_t handles (or 0) for lsm_compact_timed; `remap` = int64 [n_files]
    table of new pointer bases for lsm_compact_remap; `fences` = int64 [>= ceil(capacity / fence_stride), 4]
    that receives the fence index of the result (its first ceil(n_out / fence_stride) rows); `key_hashes` = int64
    [>= capacity] that receives the filter hash of every output key (for lsm_build_bloom_hashed)."""
    L = _load()
    runs = [_dev(r, "run") for r in runs]
    total = sum(int(r.shape[0]) for r in runs)
    dev = runs[0].device if runs else torch.device("cuda")
    if out is None:
        out = torch.empty((max(total, 1), 8), dtype=torch.int64, device=dev)
    if n_out is None:
        n_out = torch.empty(1, dtype=torch.int64, device=dev)
    if workspace is None:
        need = lsm_compact_workspace_bytes([int(r.shape[0]) for r in runs]) if runs else 0
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    rd = (_Run * max(1, len(runs)))(*[_Run(r.data_ptr(), int(r.shape[0])) for r in runs])
    od = _Out(_dev(out, "out").data_ptr(), int(out.shape[0]), _count(n_out, "n_out").data_ptr(),
              _dev(fences, "fences").data_ptr() if fences is not None else None, fence_stride if fences is not None else 0,
              _dev(key_hashes, "key hashes").data_ptr() if key_hashes is not None else None)
    if key_hashes is not None and key_hashes.numel() < out.shape[0]:
        raise ValueError("key_hashes is too short for the output capacity")
    if fences is not None and fence_stride > 0 and fences.shape[0] * fence_stride < out.shape[0]:
        raise ValueError("fences is too short for the output capacity")
    ws_ptr, ws_bytes = _dev(workspace, "workspace").data_ptr(), workspace.numel() * workspace.element_size()
    if remap is not None:
        rm = _Remap(_dev(remap, "remap table").data_ptr(), int(remap.shape[0]))
        ev = _CompactEvents(*[C.c_void_p(e or None) for e in events]) if events is not None else None
        rc = L.lsm_compact_remap(rd, len(runs), flags, C.byref(od), ws_ptr, ws_bytes, _stream_ptr(stream), C.byref(rm),
                                 C.byref(ev) if ev is not None else None)
    elif events is None:
        rc = L.lsm_compact(rd, len(runs), flags, C.byref(od), ws_ptr, ws_bytes, _stream_ptr(stream))
    else:
        ev = _CompactEvents(*[C.c_void_p(e or None) for e in events])
        rc = L.lsm_compact_timed(rd, len(runs), flags, C.byref(od), ws_ptr, ws_bytes, _stream_ptr(stream), C.byref(ev))
    if rc != 0:
        raise LsmError(rc, "lsm_compact")
    return out, n_out


class CompactCall:
    """A reusable argument block for lsm_compact on GPU tensors: the descriptors are filled in place from call to call
    instead of being built anew (a driver that issues thousands of small compactions spends more time building them than
    the kernels run).  The tensors are taken as they are (the library checks pointers, alignment and sizes); returns the
    library's status code."""

    def __init__(self):
        self._lib = _load()
        self._runs = (_Run * LSM_MAX_RUNS)()
        self._out = _Out()
        self._out_ref = C.byref(self._out)

    def __call__(self, runs: Sequence[torch.Tensor], flags: int, out: torch.Tensor, n_out: torch.Tensor,
                 fences: torch.Tensor, fence_stride: int, workspace: torch.Tensor, stream=None) -> int:
        rd = self._runs
        for j, r in enumerate(runs):
            rd[j].entries = r.data_ptr()
            rd[j].n = r.shape[0]
        od = self._out
        od.entries, od.capacity, od.n_out = out.data_ptr(), out.shape[0], n_out.data_ptr()
        od.fence_keys, od.fence_stride = fences.data_ptr(), fence_stride
        return self._lib.lsm_compact(rd, len(runs), flags, self._out_ref, workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))


def lsm_compact_static(runs: Sequence[torch.Tensor], flags: int, out: torch.Tensor, n_out: torch.Tensor, stream=None,
                       fences: Optional[torch.Tensor] = None, fence_stride: int = 64,
                       key_hashes: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """lsm_compact on the library's own static scratch: nothing is allocated, here or in the library, so the caller
    passes every buffer (out int64 [capacity, 8], n_out int64 [1])."""
    runs = [_dev(r, "run") for r in runs]
    rd = (_Run * max(1, len(runs)))(*[_Run(r.data_ptr(), int(r.shape[0])) for r in runs])
    od = _Out(_dev(out, "out").data_ptr(), int(out.shape[0]), _dev(n_out, "n_out").data_ptr(),
              _dev(fences, "fences").data_ptr() if fences is not None else None, fence_stride if fences is not None else 0,
              _dev(key_hashes, "key hashes").data_ptr() if key_hashes is not None else None)
    rc = _load().lsm_compact_static(rd, len(runs), flags, C.byref(od), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_compact_static")
    return out, n_out


def lsm_flush_buffer(buffer: torch.Tensor, out: Optional[torch.Tensor] = None, n_out: Optional[torch.Tensor] = None,
                     fences: Optional[torch.Tensor] = None, fence_stride: int = 64, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    """The write buffer (int64 [n, 8], entries in the order written) as a sorted run; returns (out, n_out) like lsm_compact."""
    L = _load()
    n = int(_dev(buffer, "buffer").shape[0])
    if out is None:
        out = torch.empty((max(n, 1), 8), dtype=torch.int64, device=buffer.device)
    if n_out is None:
        n_out = torch.empty(1, dtype=torch.int64, device=buffer.device)
    ws = torch.empty(max(int(L.lsm_flush_workspace_bytes(n)), 4), dtype=torch.uint8, device=buffer.device)
    od = _Out(_dev(out, "out").data_ptr(), int(out.shape[0]), _dev(n_out, "n_out").data_ptr(),
              _dev(fences, "fences").data_ptr() if fences is not None else None, fence_stride if fences is not None else 0)
    rc = L.lsm_flush_buffer(buffer.data_ptr(), n, C.byref(od), ws.data_ptr(), ws.numel(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_flush_buffer")
    return out, n_out


def lsm_build_fences(run: torch.Tensor, stride: int = 64, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """fence[i] = key of entry i*stride; returns int64 [ceil(n/stride), 4]."""
    L = _load()
    n = int(_dev(run, "run").shape[0])
    n_f = (n + stride - 1) // stride if stride > 0 else 0
    if out is None:
        out = torch.empty((n_f, 4), dtype=torch.int64, device=run.device)
    rd = _Run(run.data_ptr(), n)
    rc = L.lsm_build_fences(C.byref(rd), stride, _dev(out, "fences").data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_build_fences")
    return out


def lsm_bloom_blocks(n: int, bits_per_key: int = 16) -> int:
    return int(_load().lsm_bloom_blocks(n, bits_per_key))


def lsm_build_bloom(run: torch.Tensor, bits_per_key: int = 16, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Bloom filter of a run; returns int32 [n_blocks, 4] (one 16-byte block per row)."""
    L = _load()
    n = int(_dev(run, "run").shape[0])
    if out is None:
        out = torch.empty((lsm_bloom_blocks(n, bits_per_key), 4), dtype=torch.int32, device=run.device)
    rd = _Run(run.data_ptr(), n)
    rc = L.lsm_build_bloom(C.byref(rd), _dev(out, "bloom filter").data_ptr(), int(out.shape[0]), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_build_bloom")
    return out


def lsm_bloom_workspace_bytes(n: int, n_blocks: int) -> int:
    return int(_load().lsm_bloom_workspace_bytes(n, n_blocks))


def lsm_hash_keys(run: torch.Tensor, out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """The filter hash of every key of a run; returns int64 [n]."""
    n = int(_dev(run, "run").shape[0])
    if out is None:
        out = torch.empty(n, dtype=torch.int64, device=run.device)
    rd = _Run(run.data_ptr(), n)
    rc = _load().lsm_hash_keys(C.byref(rd), _dev(out, "key hashes").data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_hash_keys")
    return out


def lsm_build_bloom_hashed(hashes: torch.Tensor, n_blocks: int, out: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Bloom filter of the keys whose hashes are given (int64 [n], from lsm_hash_keys or lsm_compact's key_hashes);
    returns int32 [n_blocks, 4], the same bytes as lsm_build_bloom on the run."""
    L = _load()
    n = int(_dev(hashes, "key hashes").shape[0])
    if out is None:
        out = torch.empty((n_blocks, 4), dtype=torch.int32, device=hashes.device)
    need = int(L.lsm_bloom_workspace_bytes(n, int(out.shape[0])))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=hashes.device)
    rc = L.lsm_build_bloom_hashed(hashes.data_ptr(), n, _dev(out, "bloom filter").data_ptr(), int(out.shape[0]),
                                  _dev(workspace, "workspace").data_ptr(), workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_build_bloom_hashed")
    return out


def lsm_hash_index_buckets(n: int) -> int:
    return int(_load().lsm_hash_index_buckets(n))


def lsm_hash_index_workspace_bytes(n: int) -> int:
    return int(_load().lsm_hash_index_workspace_bytes(n))


def lsm_build_hash_index(hashes: torch.Tensor, out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                         stream=None) -> torch.Tensor:
    """Hash index of the run whose keys' hashes are given in run order (int64 [n], from lsm_hash_keys or lsm_compact's
    key_hashes); returns int64 [n_buckets, 8]."""
    L = _load()
    n = int(_dev(hashes, "key hashes").shape[0])
    if out is None:
        out = torch.empty((int(L.lsm_hash_index_buckets(n)), 8), dtype=torch.int64, device=hashes.device)
    if workspace is None:
        workspace = torch.empty(max(int(L.lsm_hash_index_workspace_bytes(n)), 256), dtype=torch.uint8, device=hashes.device)
    rc = L.lsm_build_hash_index(hashes.data_ptr(), n, _dev(out, "hash index").data_ptr(), _dev(workspace, "workspace").data_ptr(),
                                workspace.numel(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_build_hash_index")
    return out


def lsm_build_bloom_batch(runs: Sequence[torch.Tensor], bits_per_key: int = 16, stream=None) -> List[torch.Tensor]:
    """Bloom filters of several runs in one call; returns one int32 [n_blocks_j, 4] tensor per run (slices of one
    allocation)."""
    L = _load()
    if not runs:
        return []
    blocks = [lsm_bloom_blocks(int(_dev(r, "run").shape[0]), bits_per_key) for r in runs]
    all_f = torch.empty((sum(blocks), 4), dtype=torch.int32, device=runs[0].device)
    outs, at = [], 0
    for b in blocks:
        outs.append(all_f[at:at + b])
        at += b
    rd = (_Run * len(runs))(*[_Run(r.data_ptr(), int(r.shape[0])) for r in runs])
    fp = (C.c_void_p * len(runs))(*[o.data_ptr() for o in outs])
    nb = (C.c_uint64 * len(runs))(*blocks)
    rc = L.lsm_build_bloom_batch(rd, fp, nb, len(runs), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_build_bloom_batch")
    return outs


@dataclass
class TreeRun:
    run: torch.Tensor      # int64 [n, 8]
    fences: torch.Tensor   # int64 [ceil(n/stride), 4]
    stride: int = 64
    level: int = 0
    bloom: Optional[torch.Tensor] = None  # int32 [n_blocks, 4] from lsm_build_bloom, or None
    index: Optional[torch.Tensor] = None  # int64 [n_buckets, 8] from lsm_build_hash_index, or None


def _tree_descriptor(tree: Sequence[TreeRun]):
    tr = (_TreeRun * max(1, len(tree)))()
    for i, t in enumerate(tree):
        tr[i].run = _Run(_dev(t.run, "tree run").data_ptr(), int(t.run.shape[0]))
        tr[i].fence = _Fence(_dev(t.fences, "fences").data_ptr(), int(t.fences.shape[0]), t.stride)
        if t.bloom is not None:
            tr[i].bloom = _Bloom(_dev(t.bloom, "bloom filter").data_ptr(), int(t.bloom.shape[0]))
        tr[i].level = t.level
        if t.index is not None:
            tr[i].index = _HashIndex(_dev(t.index, "hash index").data_ptr(), int(t.index.shape[0]))
    return _Tree(tr, len(tree)), tr  # tr must outlive the call


def lsm_probe_length(qkeys: torch.Tensor, n_blocks: torch.Tensor, tree: Sequence[TreeRun],
                     hit_len: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Length of the longest cached prefix of every request by a search over the prefix length
    (prefix-closed data only; see the header)."""
    L = _load()
    _dev(qkeys, "qkeys")
    n_req, max_blocks = int(qkeys.shape[0]), int(qkeys.shape[1])
    if hit_len is None:
        hit_len = torch.empty(n_req, dtype=torch.int32, device=qkeys.device)
    td, _keep = _tree_descriptor(tree)
    qd = _Queries(qkeys.data_ptr(), _dev(n_blocks, "n_blocks").data_ptr(), n_req, max_blocks)
    rc = L.lsm_probe_length(C.byref(qd), C.byref(td), _dev(hit_len, "hit_len").data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_probe_length")
    return hit_len


def lsm_range_bounds(tree: Sequence[TreeRun], lo_key: bytes, hi_key: bytes, stream=None) -> torch.Tensor:
    """int64 [n_runs, 2]: entries of every run below lo_key and below hi_key."""
    L = _load()
    assert len(lo_key) == 32 and len(hi_key) == 32
    out = torch.zeros((len(tree), 2), dtype=torch.int64, device=tree[0].run.device if tree else "cuda")
    td, _keep = _tree_descriptor(tree)
    rc = L.lsm_range_bounds(C.byref(td), lo_key, hi_key, out.data_ptr(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_range_bounds")
    return out


LSM_RANGE_OVERFLOW = 0xFFFFFFFF
LSM_RANGE_MAX_ENTRIES = 2048


def lsm_range_scan(tree: Sequence[TreeRun], lo_keys: torch.Tensor, hi_keys: torch.Tensor, max_entries: int = 256,
                   entries: Optional[torch.Tensor] = None, counts: Optional[torch.Tensor] = None, stream=None
                   ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Live content of the key ranges [lo_keys[i], hi_keys[i]) (int64 [n, 4] key tensors on the GPU).  Returns
    (entries int64 [n, max_entries, 8], counts int64 [n]); counts[i] == LSM_RANGE_OVERFLOW marks a range that did not
    fit (more than 2048 entries in its pieces, or more than max_entries results)."""
    L = _load()
    n = int(_dev(lo_keys, "lo_keys").shape[0])
    assert tuple(_dev(hi_keys, "hi_keys").shape) == tuple(lo_keys.shape) and lo_keys.shape[1] == 4
    dev = lo_keys.device
    if entries is None:
        entries = torch.empty((n, max_entries, 8), dtype=torch.int64, device=dev)
    raw = torch.empty(n, dtype=torch.int32, device=dev) if counts is None else counts
    td, _keep = _tree_descriptor(tree)
    rd = _Ranges(lo_keys.data_ptr(), hi_keys.data_ptr(), n, max_entries)
    od = _RangeOut(_dev(entries, "entries").data_ptr(), _dev(raw, "counts").data_ptr())
    rc = L.lsm_range_scan(C.byref(rd), C.byref(td), C.byref(od), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_range_scan")
    return entries, (raw.to(torch.int64) & 0xFFFFFFFF) if counts is None else raw


def lsm_compact_batch(jobs: Sequence[Tuple[Sequence[torch.Tensor], int]], stream=None, fence_stride: int = 0):
    """Many independent small compactions in one call.  jobs = [(runs, flags), ...].  Returns (outs, n_out): outs[j] is
    int64 [capacity_j, 8] (a slice of one allocation), n_out int64 [n_jobs] on the device.  With fence_stride > 0 the
    fence index of every output is written in the same pass and (outs, n_out, fences) is returned: fences[j] is int64
    [ceil(capacity_j / fence_stride), 4], of which the first ceil(n_out[j] / fence_stride) rows are meaningful."""
    L = _load()
    n_jobs = len(jobs)
    dev = next((r.device for runs, _ in jobs for r in runs), torch.device("cuda"))
    totals = [sum(int(r.shape[0]) for r in runs) for runs, _ in jobs]
    out_all = torch.empty((max(sum(totals), 1), 8), dtype=torch.int64, device=dev)
    n_out = torch.empty(max(n_jobs, 1), dtype=torch.int64, device=dev)
    outs, keep, jd, at = [], [], (_CompactJob * max(1, n_jobs))(), 0
    fences, f_at = [], 0
    if fence_stride > 0:
        f_rows = [(t + fence_stride - 1) // fence_stride for t in totals]
        fence_all = torch.empty((max(sum(f_rows), 1), 4), dtype=torch.int64, device=dev)
    for j, ((runs, flags), total) in enumerate(zip(jobs, totals)):
        rd = (_Run * max(1, len(runs)))(*[_Run(_dev(r, "run").data_ptr(), int(r.shape[0])) for r in runs])
        keep.append(rd)
        outs.append(out_all[at:at + total])
        jd[j].runs, jd[j].n_runs, jd[j].flags = rd, len(runs), flags
        jd[j].out = _Out(out_all.data_ptr() + at * 64, total, n_out.data_ptr() + 8 * j, None, 0)
        if fence_stride > 0:
            fences.append(fence_all[f_at:f_at + f_rows[j]])
            jd[j].out.fence_keys, jd[j].out.fence_stride = fence_all.data_ptr() + f_at * 32, fence_stride
            f_at += f_rows[j]
        at += total
    need = int(L.lsm_compact_batch_workspace_bytes(jd, n_jobs)) if n_jobs else 0
    if n_jobs and need == 0:
        raise LsmError(-2, "lsm_compact_batch_workspace_bytes")
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    rc = L.lsm_compact_batch(jd, n_jobs, ws.data_ptr(), ws.numel(), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_compact_batch")
    return (outs, n_out[:n_jobs], fences) if fence_stride > 0 else (outs, n_out[:n_jobs])


def lsm_probe(qkeys: torch.Tensor, n_blocks: torch.Tensor, tree: Sequence[TreeRun],
              hit_len: Optional[torch.Tensor] = None, hits: Optional[torch.Tensor] = None, stream=None
              ) -> Tuple[torch.Tensor, torch.Tensor]:
    """Longest cached prefix of every request against `tree` (runs newest -> oldest)."""
    L = _load()
    _dev(qkeys, "qkeys")
    n_req, max_blocks = int(qkeys.shape[0]), int(qkeys.shape[1])
    if hit_len is None:
        hit_len = torch.empty(n_req, dtype=torch.int32, device=qkeys.device)
    if hits is None:
        hits = torch.empty((n_req, max_blocks, 2), dtype=torch.int64, device=qkeys.device)
    td, _keep = _tree_descriptor(tree)
    qd = _Queries(qkeys.data_ptr(), _dev(n_blocks, "n_blocks").data_ptr(), n_req, max_blocks)
    hd = _Hits(_dev(hit_len, "hit_len").data_ptr(), _dev(hits, "hits").data_ptr())
    rc = L.lsm_probe(C.byref(qd), C.byref(td), C.byref(hd), _stream_ptr(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_probe")
    return hit_len, hits


def _policy_input(w, s, r, z, n_entries, buffer_entries, B, p, d) -> _PolicyInput:
    return _PolicyInput(w, s, r, z, n_entries, buffer_entries, B, p, d)


def lsm_policy_levels(n_entries: int, buffer_entries: int, T: int) -> int:
    return int(_load().lsm_policy_levels(n_entries, buffer_entries, T))


def lsm_policy_cost(w, s, r, z, n_entries, buffer_entries, T, K, B, p, d) -> float:
    pin = _policy_input(w, s, r, z, n_entries, buffer_entries, B, p, d)
    return float(_load().lsm_policy_cost(C.byref(pin), T, K))


def lsm_policy_filter_fpr(bits_per_key: int) -> float:
    return float(_load().lsm_policy_filter_fpr(bits_per_key))


def lsm_policy_choose(w, s, r, z, n_entries, buffer_entries, t_min, t_max, B, p, d) -> Tuple[int, int]:
    pin = _policy_input(w, s, r, z, n_entries, buffer_entries, B, p, d)
    bt, bk = C.c_uint32(0), C.c_uint32(0)
    rc = _load().lsm_policy_choose(C.byref(pin), t_min, t_max, C.byref(bt), C.byref(bk))
    if rc != 0:
        raise LsmError(rc, "lsm_policy_choose")
    return int(bt.value), int(bk.value)


class LsmDriver:
    """lsm_driver_*: the library's own host driver of one tree (levels, controller, lazy transition; see the header).
    The driver works on the stream that is current when it is created.  Tensors handed to load_run are borrowed and
    kept alive here; everything the driver creates lives in its own pool until close()."""

    def __init__(self, buffer_entries: int, size_ratio: int = 10, runs_per_level: int = 1, window_ops: int = 4096,
                 shift_threshold: float = 0.2, t_grid: Tuple[int, int] = (10, 10), page_entries: float = 64.0,
                 filter_fpr: Optional[float] = None, fence_stride: int = 64, bloom_bits: int = 0, hash_index_from: int = 0,
                 on_compaction=None, stream=None):
        L = _load()
        self._on_compaction = on_compaction   # called with (level, int64 [n, 8] copy of the output on the GPU)
        self._observer = _DriverObserver(self._observe) if on_compaction is not None else _DriverObserver()
        cfg = _DriverConfig(buffer_entries, size_ratio, runs_per_level, window_ops, shift_threshold, t_grid[0], t_grid[1],
                            page_entries, -1.0 if filter_fpr is None else filter_fpr, fence_stride, bloom_bits, hash_index_from,
                            self._observer, None)
        self._h = C.c_void_p()
        # without a GPU only the controller can be used (note_writes, note_reads, trace, target): no stream to name
        on_gpu = stream is not None or torch.cuda.is_available()
        rc = L.lsm_driver_create(C.byref(cfg), _stream_ptr(stream) if on_gpu else None, C.byref(self._h))
        if rc != 0:
            raise LsmError(rc, "lsm_driver_create")
        self._borrowed: List[torch.Tensor] = []
        self._device = torch.device("cuda", torch.cuda.current_device()) if on_gpu else None
        self._events: List[tuple] = []

    def close(self) -> None:
        if getattr(self, "_h", None):
            _load().lsm_driver_destroy(self._h)
            self._h = None
            self._borrowed = []

    def __del__(self):
        try:
            self.close()
        except Exception:   # interpreter shutdown: the library may be gone already
            pass

    def _check(self, rc: int, where: str) -> None:
        if rc != 0:
            raise LsmError(rc, where)

    def read(self, ptr: int, rows: int, cols: int, dtype=torch.int64) -> torch.Tensor:
        """A copy, on the GPU, of rows x cols elements of driver-owned device memory."""
        out = torch.empty((rows, cols), dtype=dtype, device=self._device)
        if out.numel():
            self._check(_load().lsm_driver_read(self._h, ptr, out.data_ptr(), out.numel() * out.element_size()), "lsm_driver_read")
        return out

    def _observe(self, _ctx, level, entries, n) -> None:
        self._on_compaction(int(level), self.read(entries, int(n), 8))

    def load_run(self, level: int, run: torch.Tensor) -> None:
        """Appends `run` as the oldest run of `level` (1-based); nothing is merged."""
        self._borrowed.append(_dev(run, "run"))
        self._check(_load().lsm_driver_load_run(self._h, level, run.data_ptr(), int(run.shape[0])), "lsm_driver_load_run")

    def note_writes(self, n_ops: int) -> None:
        self._check(_load().lsm_driver_note_writes(self._h, n_ops), "lsm_driver_note_writes")

    def note_reads(self, successful: int, empty: int, blocks: int) -> None:
        """Read statistics of lookups done elsewhere: counted like one probe batch."""
        self._check(_load().lsm_driver_note_reads(self._h, successful, empty, blocks), "lsm_driver_note_reads")

    def flush(self, run: torch.Tensor) -> None:
        self._check(_load().lsm_driver_flush(self._h, _dev(run, "run").data_ptr(), int(run.shape[0])), "lsm_driver_flush")

    def flush_unsorted(self, buffer: torch.Tensor) -> None:
        self._check(_load().lsm_driver_flush_unsorted(self._h, _dev(buffer, "buffer").data_ptr(), int(buffer.shape[0])),
                    "lsm_driver_flush_unsorted")

    def probe(self, qkeys: torch.Tensor, n_blocks: torch.Tensor, hit_len: Optional[torch.Tensor] = None,
              hits: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
        n_req, max_blocks = int(_dev(qkeys, "qkeys").shape[0]), int(qkeys.shape[1])
        if hit_len is None:
            hit_len = torch.empty(n_req, dtype=torch.int32, device=qkeys.device)
        if hits is None:
            hits = torch.empty((n_req, max_blocks, 2), dtype=torch.int64, device=qkeys.device)
        qd = _Queries(qkeys.data_ptr(), _dev(n_blocks, "n_blocks").data_ptr(), n_req, max_blocks)
        hd = _Hits(_dev(hit_len, "hit_len").data_ptr(), _dev(hits, "hits").data_ptr())
        self._check(_load().lsm_driver_probe(self._h, C.byref(qd), C.byref(hd)), "lsm_driver_probe")
        return hit_len, hits

    def target(self) -> Tuple[int, int]:
        t, k = C.c_uint32(0), C.c_uint32(0)
        self._check(_load().lsm_driver_target(self._h, C.byref(t), C.byref(k)), "lsm_driver_target")
        return int(t.value), int(k.value)

    def levels(self) -> List[Tuple[int, int, int]]:
        """(T, K, number of runs) of every level, level 1 first."""
        L, out = _load(), []
        for level in range(1, int(L.lsm_driver_levels(self._h)) + 1):
            t, k, n = C.c_uint32(0), C.c_uint32(0), C.c_uint32(0)
            self._check(L.lsm_driver_level(self._h, level, C.byref(t), C.byref(k), C.byref(n)), "lsm_driver_level")
            out.append((int(t.value), int(k.value), int(n.value)))
        return out

    def tree(self):
        """The runs newest -> oldest as _TreeRun descriptors (device pointers, valid until the next flush)."""
        L, n = _load(), C.c_uint32(0)
        self._check(L.lsm_driver_tree(self._h, None, 0, C.byref(n)), "lsm_driver_tree")
        runs = (_TreeRun * max(1, n.value))()
        self._check(L.lsm_driver_tree(self._h, runs, n.value, C.byref(n)), "lsm_driver_tree")
        return [runs[i] for i in range(n.value)]

    @property
    def trace(self) -> List[tuple]:
        """The driver's log as tuples: ("adopt", level, T, K), ("compact", level, runs, n_in, n_out, flags),
        ("move", level, to, n), ("probe", requests, hits, blocks), ("policy", T, K, mix rounded to 6 places, d likewise)."""
        L = _load()
        total = int(L.lsm_driver_log(self._h, 0, None, 0))
        while len(self._events) < total:
            buf = (_DriverEvent * min(total - len(self._events), 4096))()
            L.lsm_driver_log(self._h, len(self._events), buf, len(buf))
            for e in buf:
                if e.kind == 1:
                    self._events.append(("adopt", e.level, e.a, e.b))
                elif e.kind == 2:
                    self._events.append(("compact", e.level, e.a, e.n_in, e.n_out, e.b))
                elif e.kind == 3:
                    self._events.append(("move", e.level, e.a, e.n_out))
                elif e.kind == 4:
                    self._events.append(("probe", e.a, e.b, e.n_out))
                else:
                    self._events.append(("policy", e.a, e.b, tuple(round(x, 6) for x in e.mix), round(e.d, 6)))
        return self._events


def lsm_driver_flush_many(drivers: Sequence[LsmDriver], runs: Sequence[Optional[torch.Tensor]]) -> None:
    """One flush for each of several independent trees, stepped together: the compactions their cascades need at the same
    step run as one batch.  runs[i] is tree i's sorted write buffer, or None if it has nothing to flush."""
    count = len(drivers)
    if count == 0:
        return
    assert len(runs) == count
    hd = (C.c_void_p * count)(*[d._h for d in drivers])
    # an empty write buffer is still a flush (an empty run arrives): any non-null address says so, it is never read
    ptr = (C.c_void_p * count)(*[None if r is None else (_dev(r, "run").data_ptr() or 64) for r in runs])
    n = (C.c_uint64 * count)(*[0 if r is None else int(r.shape[0]) for r in runs])
    rc = _load().lsm_driver_flush_many(hd, ptr, n, count)
    if rc != 0:
        raise LsmError(rc, "lsm_driver_flush_many")
