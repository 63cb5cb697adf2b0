"""Plain replay of the adaptive controller and of the level bookkeeping it steers (test infrastructure only).

Only tests may import this module.  It shares no code with the package: it keeps its own window of operations, its
own per-level parameters and its own merge rule, and it moves numpy runs with the C checker's heap merge and
linear-scan probe (oracle/lsm_oracle.c).  What it states, in the paper's order:

Tree (section 2.2).  Writes fill a buffer of M entries that is flushed as a sorted run into level 1.  Level i (1-based)
holds at most K_i runs and at most M * T_i**i entries.  Compaction merges runs, keeps sorted order and removes
obsolete entries; tombstones are removed only when nothing lies below the output.

Controller (section 3.3).  Operation counts are kept over a sliding window; their shares are the coefficients
w (writes), s and r (both from successful reads: half each) and z (probes that find nothing) of the cost
w*W + s*S + r*R + z*Z with the operation costs of section 2.2.  When the mix has moved by more than a threshold
since the last search, every (T, K) of the grid is costed and the cheapest pair becomes the target.

Lazy transition (appendix C).  Nothing is restructured when the target changes.  A level takes over the target T
and K at the moment data next flows into it (a flushed run for level 1, a run moved down for the others).
K larger than before: the run already there stays as it is and the newcomer sits beside it.  K smaller than before:
the level holds more runs than allowed after the arrival, so they are all merged then - the same rule that bounds
the run count in steady state.  A merged run that exceeds the level's capacity moves down, where the same happens.

Readings (the paper fixes no constants):
  * an operation is one inserted sequence (write) or one probe request (read); a probe request that finds no live
    first block is an empty probe; d = mean number of blocks a successful request found;
  * statistics arrive in batches (the writes since the last event, or one probe batch); the window is the shortest
    suffix of batches that still covers `window_ops` operations, and no search is made before it is that long;
  * the mix has moved when the L1 distance of (w, s, r, z) to the mix at the last search exceeds `threshold`;
  * N of the cost model is the number of entries in the tree at the time of the search.
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from . import lsm_oracle as _o


class Level:
    """One level: its runs (index 0 = the run that arrived last) and the parameters it currently runs with."""

    def __init__(self, T: int, K: int):
        self.runs: List[np.ndarray] = []
        self.T = T
        self.K = K


class DriverOracle:
    def __init__(self, buffer_entries: int, T: int = 10, K: int = 1, window_ops: int = 4096, threshold: float = 0.2,
                 t_grid: Tuple[int, int] = (10, 10), page_entries: float = 64.0, fpr: float = 1.0,
                 choose: Optional[Callable] = None, probe_fn: Optional[Callable] = None,
                 on_compact: Optional[Callable] = None):
        self.M = int(buffer_entries)
        self.target_T, self.target_K = int(T), int(K)
        self.window_ops, self.threshold = int(window_ops), float(threshold)
        self.t_grid, self.B, self.p = t_grid, float(page_entries), float(fpr)
        self.choose = choose or _o.policy_choose
        self.probe_fn = probe_fn or _o.probe      # a test may pass a wrapper that splits the requests over threads
        self.on_compact = on_compact              # called with every compaction output (streamed comparison)
        self.levels: List[Level] = []
        self.log: List[tuple] = []
        self.batches: List[Tuple[int, int, int, int]] = []  # (writes, successful reads, empty probes, blocks found), oldest first
        self.mix_at_last_search: Optional[Tuple[float, float, float, float]] = None

    # ---------------------------------------------------------------- tree
    def install(self, level: int, runs_newest_first: Sequence) -> None:
        """Put runs into level `level` (1-based) without any merging: the starting tree."""
        self._grow(level)
        self.levels[level - 1].runs = [_o.as_run(r) for r in runs_newest_first]

    def _grow(self, level: int) -> None:
        while len(self.levels) < level:
            self.levels.append(Level(self.target_T, self.target_K))

    def entries(self) -> int:
        return sum(r.shape[0] for lv in self.levels for r in lv.runs)

    def runs_newest_first(self) -> List[np.ndarray]:
        return [r for lv in self.levels for r in lv.runs]

    def flush(self, run) -> None:
        """A sorted run from the write buffer: data flows into level 1, and onwards while levels overflow."""
        level, moving = 1, _o.as_run(run)
        while moving is not None:
            self._grow(level)
            lv = self.levels[level - 1]
            if (lv.T, lv.K) != (self.target_T, self.target_K):
                self.log.append(("adopt", level, self.target_T, self.target_K))
            lv.T, lv.K = self.target_T, self.target_K           # lazy transition: parameters change where data arrives
            lv.runs.insert(0, moving)
            moving = None
            if len(lv.runs) <= lv.K:
                break                                            # room for one more run: nothing is merged
            below_empty = all(len(x.runs) == 0 for x in self.levels[level:])
            flags = _o.FLAG_BOTTOMMOST if below_empty else 0
            n_in = sum(r.shape[0] for r in lv.runs)
            merged = _o.compact(lv.runs, flags)
            self.log.append(("compact", level, len(lv.runs), n_in, int(merged.shape[0]), flags))
            if self.on_compact is not None:
                self.on_compact(merged)
            lv.runs = []
            if merged.shape[0] > self.M * lv.T ** level:
                self.log.append(("move", level, level + 1, int(merged.shape[0])))
                moving, level = merged, level + 1
            elif merged.shape[0] > 0:
                lv.runs = [merged]

    # ---------------------------------------------------------------- operations
    def writes(self, n_sequences: int) -> None:
        self._observe(int(n_sequences), 0, 0, 0)

    def probe(self, qkeys, n_blocks):
        hit_len, hits = self.probe_fn(qkeys, n_blocks, self.runs_newest_first())
        found = hit_len[hit_len > 0]
        self.log.append(("probe", int(hit_len.shape[0]), int(found.shape[0]), int(found.sum())))
        self._observe(0, int(found.shape[0]), int(hit_len.shape[0] - found.shape[0]), int(found.sum()))
        return hit_len, hits

    def observe_reads(self, successful: int, empty: int, blocks: int) -> None:
        """Read statistics without running a probe (used by the hand-worked trace)."""
        self.log.append(("probe", successful + empty, successful, blocks))
        self._observe(0, successful, empty, blocks)

    # ---------------------------------------------------------------- controller
    def _slide(self) -> int:
        """Drop the batches that the window no longer needs; returns the operations it covers now."""
        ops = [b[0] + b[1] + b[2] for b in self.batches]
        start, covered = len(ops), 0
        while start > 0 and covered < self.window_ops:          # shortest suffix that covers window_ops operations
            start -= 1
            covered += ops[start]
        self.batches = self.batches[start:]
        return covered

    def _observe(self, wr: int, ok: int, empty: int, blocks: int) -> None:
        self.batches.append((wr, ok, empty, blocks))
        covered = self._slide()
        if covered < self.window_ops:
            return                                               # the window is not full yet
        wr_sum = sum(b[0] for b in self.batches)
        ok_sum = sum(b[1] for b in self.batches)
        empty_sum = sum(b[2] for b in self.batches)
        block_sum = sum(b[3] for b in self.batches)
        mix = (wr_sum / covered, ok_sum / covered / 2, ok_sum / covered / 2, empty_sum / covered)
        if self.mix_at_last_search is not None:
            moved = sum(abs(now - then) for now, then in zip(mix, self.mix_at_last_search))
            if moved <= self.threshold:
                return
        self.mix_at_last_search = mix
        d = block_sum / ok_sum if ok_sum else 0.0
        T, K = self.choose(mix[0], mix[1], mix[2], mix[3], max(1, self.entries()), self.M, self.t_grid[0], self.t_grid[1],
                           self.B, self.p, d)
        self.log.append(("policy", T, K, tuple(round(x, 6) for x in mix), round(d, 6)))
        self.target_T, self.target_K = T, K


def bloom_fpr(bits_per_key: int, block_bits: int = 128, bits_set: int = 6) -> float:
    """False-positive rate p (section 2.2) of the blocked filter described with lsm_bloom_t: a key sets `bits_set` bits
    of one `block_bits`-bit block; with b bits per key a block receives Poisson(block_bits / b) keys; a block that
    received n keys has each bit set with probability 1 - (1 - 1/block_bits)**(bits_set * n), and a foreign key
    passes when its `bits_set` bits (drawn independently, with repetition) are all set.  0 bits per key: no filter, p = 1."""
    if bits_per_key <= 0:
        return 1.0
    lam = block_bits / bits_per_key
    spread = 12.0 * math.sqrt(lam) + 50.0
    total = 0.0
    for n in range(max(0, int(lam - spread)), int(lam + spread) + 1):
        weight = math.exp(-lam + n * math.log(lam) - math.lgamma(n + 1))  # Poisson(n; lam)
        fill = 1.0 - (1.0 - 1.0 / block_bits) ** (bits_set * n)
        total += weight * fill ** bits_set
    return total
