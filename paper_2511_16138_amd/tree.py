"""Host driver of the LSM key index: level bookkeeping and the adaptive controller.

This sequences the library calls for a mixed workload (paper section 3.3 and appendix C):
flushed runs enter level 1, a level that holds more than K runs is compacted, a level that
outgrows its capacity M * T**level is moved down, and a sliding window of operation counts
re-tunes (T, K) through the cost model.  All index work (merging, fence building, lookups, the
cost model itself) is done by the backend = the GPU library; nothing here touches entries.

Readings of the paper used here (it gives no constants):
  * a sliding window over the last `window_ops` operations; a write operation is one inserted
    sequence, a read one probe request; reads that find nothing count as empty probes (z), the
    others are split evenly between range reads (s) and point reads (r), since the paper takes
    both coefficients from the successful reads;
  * once the window is full, the (T, K) search is re-run whenever the L1 distance between the
    window's mix and the mix at the last search exceeds `shift_threshold`;
  * lazy transition: a level adopts the current T and K the next time a run arrives at it (data
    flowing between levels).  A larger K leaves resident runs as they are (the newcomer is placed
    beside them); a smaller K merges all runs of the level at that next arrival; a new T changes
    the level's capacity M * T**level from then on;
  * p of the lookup costs is the false-positive rate of the Bloom filters the backend builds
    (lsm_policy_filter_fpr of their bits per key), 1 without filters.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Any, List, Optional, Sequence, Tuple

LSM_BOTTOMMOST = 1


@dataclass
class LevelRun:
    run: Any      # backend handle of the entries (has .shape[0] = number of entries)
    fences: Any   # backend handle of its fence index
    bloom: Any = None  # backend handle of its Bloom filter, if the backend builds them
    index: Any = None  # backend handle of its hash index, if the backend builds them

    @property
    def n(self) -> int:
        return int(self.run.shape[0])


class GpuBackend:
    """The library calls the driver needs, on torch CUDA tensors."""

    def __init__(self, fence_stride: int = 64, bloom_bits: int = 0, hash_index_from: int = 0):
        from . import binding
        self._b = binding
        self.fence_stride = fence_stride
        self.bloom_bits = bloom_bits  # bits per key of the per-run Bloom filters; 0 = none
        self.hash_index_from = hash_index_from  # runs of at least this many entries get a hash index; 0 = none

    def compact(self, runs: Sequence[Any], flags: int) -> Any:
        import torch
        runs = [r if r.is_contiguous() else r.contiguous() for r in runs]
        if len(runs) > self._b.LSM_MAX_RUNS:
            raise ValueError("too many runs for one compaction")
        total = sum(r.shape[0] for r in runs)
        device = runs[0].device
        fences = torch.empty(((total + self.fence_stride - 1) // self.fence_stride, 4), dtype=torch.int64, device=device)
        out = torch.empty((max(total, 1), 8), dtype=torch.int64, device=device)
        # one workspace for all compactions of this backend (they follow each other on one stream), grown when the library
        # says it is too small; the count goes straight to pinned host memory: one stream synchronisation, no copy
        call = getattr(self, "_call", None)
        if call is None:
            call = self._call = self._b.CompactCall()
            self._n_host = torch.empty(1, dtype=torch.int64, pin_memory=True)
            self._workspace = torch.empty(1 << 20, dtype=torch.uint8, device=device)
        rc = call(runs, flags, out, self._n_host, fences, self.fence_stride, self._workspace)
        if rc == -4:   # LSM_ERR_WORKSPACE
            need = self._b.lsm_compact_workspace_bytes([int(r.shape[0]) for r in runs])
            self._workspace = torch.empty(2 * need, dtype=torch.uint8, device=device)
            rc = call(runs, flags, out, self._n_host, fences, self.fence_stride, self._workspace)
        if rc != 0:
            raise self._b.LsmError(rc, "lsm_compact")
        torch.cuda.current_stream().synchronize()
        n = int(self._n_host.item())
        if n < 0 or n > out.shape[0]:
            raise RuntimeError("lsm_compact reported a device-side failure")
        merged = out[:n]
        # the compaction wrote the fence index of its output in the same pass: the driver takes it right after this call
        self._fused = (merged, fences[: (n + self.fence_stride - 1) // self.fence_stride]) if n > 0 else None
        return merged

    def pop_fused_fences(self, merged: Any) -> Any:
        """The fence index that the last compact() wrote for its output `merged` (None if it is not that output)."""
        fused, self._fused = getattr(self, "_fused", None), None
        return fused[1] if fused is not None and fused[0] is merged else None

    def build_fences(self, run: Any) -> Any:
        return self._b.lsm_build_fences(run.contiguous(), self.fence_stride)

    def compact_batch(self, jobs: Sequence[Tuple[Sequence[Any], int]]) -> List[LevelRun]:
        """Independent compactions (of different trees) in one library call, with the fence indices written in the same
        pass and the Bloom filters of all outputs built by one more call; the counts come back in one copy."""
        outs, n_out, fences = self._b.lsm_compact_batch([(list(runs), flags) for runs, flags in jobs], fence_stride=self.fence_stride)
        counts = n_out.cpu().tolist()
        merged, fence_of = [], []
        for out, n, f in zip(outs, counts, fences):
            if n < 0 or n > out.shape[0]:
                raise RuntimeError("lsm_compact_batch reported a device-side failure")
            merged.append(out[:n])
            fence_of.append(f[: (n + self.fence_stride - 1) // self.fence_stride])
        live = [i for i, m in enumerate(merged) if int(m.shape[0]) > 0]
        blooms = dict(zip(live, self._b.lsm_build_bloom_batch([merged[i] for i in live], self.bloom_bits))) if self.bloom_bits else {}
        return [LevelRun(m, fence_of[i] if int(m.shape[0]) > 0 else None, blooms.get(i)) for i, m in enumerate(merged)]

    def flush_buffer(self, buffer: Any) -> Any:
        out, n_out = self._b.lsm_flush_buffer(buffer.contiguous())
        return out[: int(n_out.item())]

    def build_bloom(self, run: Any, hashes: Any = None) -> Any:
        if not self.bloom_bits:
            return None
        run = run.contiguous()
        n = int(run.shape[0])
        n_blocks = self._b.lsm_bloom_blocks(n, self.bloom_bits)
        # a long run: the filter is built from the keys' hashes, sorted by block range (no atomic traffic on the filter)
        if (hashes is not None or n >= (1 << 20)) and self._b.lsm_bloom_workspace_bytes(n, n_blocks):
            return self._b.lsm_build_bloom_hashed(hashes if hashes is not None else self._b.lsm_hash_keys(run), n_blocks)
        return self._b.lsm_build_bloom(run, self.bloom_bits)

    def build_lookup(self, run: Any) -> Tuple[Any, Any]:
        """Filter and hash index of a run that has come to rest (either may be None); the keys are hashed once for both."""
        n = int(run.shape[0])
        indexed = self.hash_index_from and n >= self.hash_index_from and n <= (1 << 27)
        hashes = self._b.lsm_hash_keys(run.contiguous()) if indexed else None
        return self.build_bloom(run, hashes), (self._b.lsm_build_hash_index(hashes) if indexed else None)

    def probe(self, qkeys: Any, n_blocks: Any, tree: Sequence[LevelRun]) -> Tuple[Any, Any]:
        tr = [self._b.TreeRun(t.run, t.fences, self.fence_stride, i, t.bloom, t.index) for i, t in enumerate(tree)]
        return self._b.lsm_probe(qkeys, n_blocks, tr)

    def hit_len_to_host(self, hit_len: Any) -> List[int]:
        return hit_len.cpu().tolist()

    def policy_choose(self, w, s, r, z, n_entries, buffer_entries, t_min, t_max, B, p, d) -> Tuple[int, int]:
        return self._b.lsm_policy_choose(w, s, r, z, n_entries, buffer_entries, t_min, t_max, B, p, d)

    def filter_fpr(self) -> float:
        return self._b.lsm_policy_filter_fpr(self.bloom_bits)


@dataclass
class AdaptiveLsmTree:
    backend: Any
    buffer_entries: int                 # M
    size_ratio: int = 10                # T
    runs_per_level: int = 1             # K currently asked for by the controller
    window_ops: int = 4096
    shift_threshold: float = 0.2
    t_grid: Tuple[int, int] = (10, 10)
    page_entries: float = 64.0          # B
    filter_fpr: Optional[float] = None  # p; None = ask the backend (1 when it builds no Bloom filters)
    levels: List[List[LevelRun]] = field(default_factory=list)   # levels[0] = level 1; runs newest first
    level_k: List[int] = field(default_factory=list)             # K each level is currently run with
    level_t: List[int] = field(default_factory=list)             # T each level is currently run with
    trace: List[tuple] = field(default_factory=list)
    _events: Any = field(default_factory=lambda: __import__("collections").deque())  # (writes, hits, empties, blocks hit)
    _win: List[float] = field(default_factory=lambda: [0, 0, 0, 0.0])  # sums over _events
    _last_mix: Optional[Tuple[float, float, float, float]] = None

    def __post_init__(self) -> None:
        if self.filter_fpr is None:
            fpr = getattr(self.backend, "filter_fpr", None)
            self.filter_fpr = float(fpr()) if fpr else 1.0

    # ------------------------------------------------------------------ structure
    def _ensure_level(self, level: int) -> None:
        while len(self.levels) <= level:
            self.levels.append([])
            self.level_k.append(self.runs_per_level)
            self.level_t.append(self.size_ratio)

    def load_level(self, level: int, runs_newest_first: Sequence[Any]) -> None:
        self._ensure_level(level)
        self.levels[level] = [self._index(r) for r in runs_newest_first]

    def _index(self, run: Any) -> LevelRun:
        """A run with the lookup structures the backend builds for it (fence index, optional Bloom filter and hash index)."""
        return self._settle(LevelRun(run, None if int(run.shape[0]) else self.backend.build_fences(run)))

    def capacity(self, level: int) -> int:
        return self.buffer_entries * self.level_t[level] ** (level + 1)

    def total_entries(self) -> int:
        return sum(r.n for lv in self.levels for r in lv)

    def tree_runs(self) -> List[LevelRun]:
        return [r for lv in self.levels for r in lv]

    def _settle(self, lr: LevelRun) -> LevelRun:
        """A run that comes to rest in a level gets whatever lookup structure it still lacks.  (Runs that are merged
        away at once - a flushed run arriving at a full level, a run moved down onto another - never get any.)"""
        if lr.n == 0:
            if lr.fences is None:
                lr.fences = self.backend.build_fences(lr.run)   # an empty index, so that lookups can name the run
            return lr
        if lr.fences is None:
            lr.fences = self.backend.build_fences(lr.run)
        build_lookup = getattr(self.backend, "build_lookup", None)
        if lr.bloom is None and lr.index is None and build_lookup:
            lr.bloom, lr.index = build_lookup(lr.run)
        elif lr.index is None and build_lookup and getattr(self.backend, "hash_index_from", 0):
            lr.index = build_lookup(lr.run)[1]   # a run of a batch already has its filter
        return lr

    def flush(self, run: Any) -> None:
        """A sorted run from the write buffer enters level 1."""
        self._arrive(0, LevelRun(run, None))

    def flush_unsorted(self, buffer: Any) -> None:
        """The write buffer as it was filled (any order, repeated keys): sorted and deduplicated by the backend first."""
        self.flush(self.backend.flush_buffer(buffer))

    def _arrive(self, level: int, newcomer: LevelRun) -> None:
        """A run arrives at a level; the compactions this triggers are run one after the other."""
        steps = self._arrive_steps(level, newcomer)
        try:
            runs, flags = next(steps)
            while True:
                merged = self.backend.compact(runs, flags)
                pop = getattr(self.backend, "pop_fused_fences", None)
                runs, flags = steps.send(LevelRun(merged, pop(merged) if pop else None))
        except StopIteration:
            pass

    def _arrive_steps(self, level: int, newcomer: LevelRun):
        """The same cascade as a generator: yields (runs, flags) for every compaction it needs and is sent the merged
        run with its lookup structures (a LevelRun), so that a caller who steps several trees together can run their
        compactions - and build their indices - as one batch."""
        while newcomer is not None:
            self._ensure_level(level)
            if (self.level_t[level], self.level_k[level]) != (self.size_ratio, self.runs_per_level):
                self.trace.append(("adopt", level + 1, self.size_ratio, self.runs_per_level))
            # lazy transition: the level takes the current parameters when data flows into it
            self.level_t[level], self.level_k[level] = self.size_ratio, self.runs_per_level
            lv = self.levels[level]
            lv.insert(0, newcomer)
            newcomer = None
            if len(lv) <= self.level_k[level]:
                lv[0] = self._settle(lv[0])
                return
            deeper_empty = all(len(x) == 0 for x in self.levels[level + 1:])
            flags = LSM_BOTTOMMOST if deeper_empty else 0
            n_in = sum(r.n for r in lv)
            merged = yield [r.run for r in lv], flags
            self.trace.append(("compact", level + 1, len(lv), n_in, merged.n, flags))
            self.levels[level] = []
            if merged.n > self.capacity(level):
                self.trace.append(("move", level + 1, level + 2, merged.n))
                newcomer, level = merged, level + 1
            elif merged.n > 0:
                self.levels[level] = [self._settle(merged)]

    # ------------------------------------------------------------------ operations and controller
    def _count(self, writes: int, hits: int, empties: int, blocks: float) -> None:
        self._events.append((writes, hits, empties, blocks))
        for i, v in enumerate((writes, hits, empties, blocks)):
            self._win[i] += v
        # slide: drop the oldest events while the rest still covers window_ops operations
        while len(self._events) > 1:
            w0, h0, e0, b0 = self._events[0]
            if self._win[0] + self._win[1] + self._win[2] - (w0 + h0 + e0) < self.window_ops:
                break
            self._events.popleft()
            for i, v in enumerate((w0, h0, e0, b0)):
                self._win[i] -= v
        self._maybe_retune()

    def note_writes(self, n_ops: int) -> None:
        self._count(n_ops, 0, 0, 0.0)

    def probe(self, qkeys: Any, n_blocks: Any) -> Tuple[Any, Any]:
        hit_len, hits = self.backend.probe(qkeys, n_blocks, self.tree_runs())
        lens = self.backend.hit_len_to_host(hit_len)
        hit = [x for x in lens if x > 0]
        self.trace.append(("probe", len(lens), len(hit), int(sum(hit))))
        self._count(0, len(hit), len(lens) - len(hit), float(sum(hit)))
        return hit_len, hits

    def _maybe_retune(self) -> None:
        writes, hits, empties, blocks = self._win
        total = writes + hits + empties
        if total < self.window_ops:
            return
        mix = (writes / total, hits / total / 2, hits / total / 2, empties / total)  # w, s, r, z
        d = blocks / hits if hits else 0.0
        if self._last_mix is not None and sum(abs(a - b) for a, b in zip(mix, self._last_mix)) <= self.shift_threshold:
            return
        self._last_mix = mix
        T, K = self.backend.policy_choose(mix[0], mix[1], mix[2], mix[3], max(1, self.total_entries()), self.buffer_entries,
                                          self.t_grid[0], self.t_grid[1], self.page_entries, self.filter_fpr, d)
        self.trace.append(("policy", T, K, tuple(round(x, 6) for x in mix), round(d, 6)))
        self.size_ratio, self.runs_per_level = T, K


class ShardedLsmTrees:
    """Several independent trees (key-range shards of one index, or one index per tenant) stepped together.  The
    flush / compaction cycles of the small upper levels (section 2.2) of different trees do not depend on each other,
    so the compactions that one round of flushes triggers are handed to the backend as one batch, and so are the
    compactions of the next step of their cascades, until every tree is settled.  Each tree keeps its own controller."""

    def __init__(self, trees: Sequence[AdaptiveLsmTree], backend: Any):
        self.trees, self.backend = list(trees), backend

    def flush_all(self, runs: Sequence[Any]) -> None:
        """runs[i]: a sorted run from tree i's write buffer, or None if tree i has nothing to flush now."""
        active = []
        for tree, run in zip(self.trees, runs):
            if run is None:
                continue
            steps = tree._arrive_steps(0, LevelRun(run, None))  # indexed only if it comes to rest (level 1 empty)
            try:
                active.append((steps, next(steps)))
            except StopIteration:
                pass
        while active:
            merged = self.backend.compact_batch([job for _, job in active])  # LevelRuns: merged run, fences, filter
            still = []
            for (steps, _), m in zip(active, merged):
                try:
                    still.append((steps, steps.send(m)))
                except StopIteration:
                    pass
            active = still


def run_mixed_trace(tree: AdaptiveLsmTree, trace, on_probe=None, on_compaction=None, shuffle_writes=None) -> None:
    """Replay a workloads.lsm.MixedTrace: flushes and probe batches in time order."""
    for (kind, i, _phase), n_writes in zip(trace.events, trace.write_ops_between):
        if n_writes:
            tree.note_writes(n_writes)
        if kind == "flush":
            before = len(tree.trace)
            if shuffle_writes is not None:  # hand the buffer over in the order the generator "wrote" it, not sorted
                tree.flush_unsorted(trace.flush_runs[i][shuffle_writes(i, int(trace.flush_runs[i].shape[0]))])
            else:
                tree.flush(trace.flush_runs[i])
            if on_compaction is not None:
                for ev in tree.trace[before:]:
                    on_compaction(ev)
        else:
            q, nb = trace.probe_batch(i)
            out = tree.probe(q, nb)
            if on_probe is not None:
                on_probe(i, q, nb, out)


def range_scan(tree_runs: Sequence[Any], lo_key: bytes, hi_key: bytes) -> Any:
    """Range lookup (section 2.2 "Range Lookups"; appendix B, get_batch): the live entries with lo_key <= key < hi_key,
    newest version of each, ascending.  Two library calls: the bounds of the range in every run, then one last-level
    compaction of the slices.  tree_runs: binding.TreeRun objects, newest run first."""
    from . import binding as b
    bounds = b.lsm_range_bounds(tree_runs, lo_key, hi_key).cpu().tolist()
    slices = [t.run[lo:hi] for t, (lo, hi) in zip(tree_runs, bounds)]
    if not slices:
        return None
    out, n_out = b.lsm_compact(slices, b.LSM_BOTTOMMOST)
    n = int(n_out.item())
    if n < 0 or n > out.shape[0]:
        raise RuntimeError("lsm_compact reported a device-side failure")
    return out[:n]


def range_scan_batch(tree_runs: Sequence[Any], lo_keys: Any, hi_keys: Any, max_entries: int = 256) -> List[Any]:
    """The range lookups of a get_batch in one library call (appendix B): for every range [lo_keys[i], hi_keys[i]) the
    live entries, newest version of each, ascending (their value pointers and lengths are the read list for the tensor
    files).  lo_keys, hi_keys: int64 [n, 4] key tensors on the GPU.  A range that does not fit its slot is redone alone
    with range_scan."""
    from . import binding as b
    entries, counts = b.lsm_range_scan(tree_runs, lo_keys, hi_keys, max_entries)
    counts = counts.cpu().tolist()
    out = []
    for i, c in enumerate(counts):
        if c == b.LSM_RANGE_OVERFLOW:
            lo, hi = (bytes(k.cpu().numpy().tobytes()) for k in (lo_keys[i], hi_keys[i]))
            out.append(range_scan(tree_runs, lo, hi))
        else:
            out.append(entries[i, :c])
    return out
