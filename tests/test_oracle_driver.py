"""The plain adaptive driver (oracle/lsm_driver_oracle.py) against things other than itself: the hand-worked trace
under tests/golden/ (level contents, compactions, transitions of K and the policy decisions with their arithmetic
written out), closed forms of the controller, and planted mistakes that the trace must notice."""
import math
import os
import re

import numpy as np
import pytest

import brute

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "adaptive_driver_trace.txt")


def key_of(k: int) -> bytes:
    return int(k).to_bytes(32, "big")


def parse_keys(tokens):
    """'1-4', '7', '!6' -> list of (key number, is tombstone)."""
    out = []
    for t in tokens:
        tomb = t.startswith("!")
        t = t.lstrip("!")
        if "-" in t:
            a, b = t.split("-")
            out += [(k, tomb) for k in range(int(a), int(b) + 1)]
        else:
            out.append((int(t), tomb))
    return out


class Script:
    """The golden file as a list of steps: (command, argument tokens, expected log records, expected tree or None)."""

    def __init__(self, path):
        self.config, self.steps, self.newest = {}, [], []
        for line in open(path):
            line = line.split("#")[0].strip()
            if not line:
                continue
            word, rest = line.split()[0], line.split()[1:]
            if word == "config":
                self.config = dict(t.split("=") for t in rest)
            elif word in ("writes", "reads", "flush"):
                self.steps.append([word, rest, [], None])
            elif word == "log":
                self.steps[-1][2].append(self.record(rest))
            elif word == "tree":
                self.steps[-1][3] = self.tree(" ".join(rest))
            elif word == "newest":
                self.newest.append((int(rest[0][1:-1]), [tuple(map(int, t.split("@"))) for t in rest[1:]]))
            else:
                raise ValueError(line)

    @staticmethod
    def record(tokens):
        kind, f = tokens[0], dict(t.split("=") for t in tokens[1:])
        if kind == "compact":
            return ("compact", int(f["level"]), int(f["runs"]), int(f["in"]), int(f["out"]), int(f["last"]))
        if kind == "move":
            return ("move", int(f["from"]), int(f["to"]), int(f["n"]))
        if kind == "adopt":
            return ("adopt", int(f["level"]), int(f["T"]), int(f["K"]))
        if kind == "probe":
            return ("probe", int(f["requests"]), int(f["found"]), int(f["blocks"]))
        if kind == "policy":
            return ("policy", int(f["T"]), int(f["K"]), tuple(float(x) for x in f["mix"].split(",")), float(f["d"]))
        raise ValueError(kind)

    @staticmethod
    def tree(text):
        levels = {}
        for part in text.split(";"):
            name, runs = part.split(":")
            levels[int(name.strip()[1:])] = [parse_keys(r.split()) for r in runs.split("|") if r.strip()]
        return levels


def make_driver(oracle, cfg, **over):
    from oracle import lsm_driver_oracle as drv
    tg = tuple(int(x) for x in cfg["tgrid"].split(","))
    kw = dict(buffer_entries=int(cfg["M"]), T=int(cfg["T"]), K=int(cfg["K"]), window_ops=int(cfg["window"]),
              threshold=float(cfg["threshold"]), t_grid=tg, page_entries=float(cfg["B"]), fpr=float(cfg["p"]))
    kw.update(over)
    return drv.DriverOracle(**kw)


def replay(oracle, script, driver, check=True):
    """Feed the script to the driver; with check, compare log and tree after every step.  Returns the mismatches."""
    seq, bad = 0, []
    for step, (cmd, args, want_log, want_tree) in enumerate(script.steps):
        before = len(driver.log)
        if cmd == "writes":
            driver.writes(int(args[0]))
        elif cmd == "reads":
            driver.observe_reads(int(args[0]), int(args[1]), int(args[2]))
        else:
            raw = []
            for k, tomb in parse_keys(args):
                seq += 1
                raw.append(brute.pack_entry(key_of(k), seq, brute.TOMBSTONE if tomb else brute.PUT, vptr=seq * 16, vlen=640))
            raw.sort(key=lambda e: e[:32])
            driver.flush(brute.run_from_raw(raw))
        got_log = driver.log[before:]
        if got_log != want_log:
            bad.append((step, cmd, args, "log", got_log, want_log))
        if want_tree is not None:
            got_tree = {}
            for i, lv in enumerate(driver.levels):
                runs = []
                for r in lv.runs:
                    rec = r.view(oracle.ENTRY_DTYPE).reshape(-1)
                    runs.append([(int.from_bytes(bytes(e["key"]), "big"), int(e["type"]) == 1) for e in rec])
                got_tree[i + 1] = runs
            for lvl in set(got_tree) | set(want_tree):
                if got_tree.get(lvl, []) != want_tree.get(lvl, []):
                    bad.append((step, cmd, args, "tree", got_tree, want_tree))
                    break
        if check:
            assert not bad, bad[0]
    return bad


def test_hand_worked_trace(oracle):
    script = Script(GOLDEN)
    assert sum(1 for s in script.steps if s[0] == "flush") == 12
    driver = make_driver(oracle, script.config)
    replay(oracle, script, driver)
    kinds = [r[0] for r in driver.log]
    ks = [r[2] for r in driver.log if r[0] == "policy"]
    assert 2 in ks and 1 in ks and ks[0] == 2 and ks[-1] == 2   # K goes up, down and up again
    assert kinds.count("adopt") == 3 and kinds.count("move") == 2
    for level, pairs in script.newest:
        (run,) = driver.levels[level - 1].runs
        rec = run.view(oracle.ENTRY_DTYPE).reshape(-1)
        seq_of = {int.from_bytes(bytes(e["key"]), "big"): int(e["seqno"]) for e in rec}
        for k, s in pairs:
            assert seq_of[k] == s, (level, k, seq_of[k], s)
    # lookups through the driver see the newest version wherever it lives, and no deleted key
    q = np.zeros((3, 1, 32), dtype=np.uint8)
    for i, k in enumerate((5, 6, 1)):
        q[i, 0] = np.frombuffer(key_of(k), dtype=np.uint8)
    hit_len, hits = driver.probe(q, np.ones(3, dtype=np.uint32))
    assert hit_len.tolist() == [1, 0, 1]
    assert int(hits[0, 0]["vptr"]) == 45 * 16 and int(hits[0, 0]["run_idx"]) == 0
    assert int(hits[2, 0]["vptr"]) == 25 * 16 and int(hits[2, 0]["run_idx"]) == 1


def test_policy_lines_of_the_trace_follow_from_the_cost_formula(oracle):
    """Every policy line of the golden file again, from the formulas of sections 2.2 and 3.3 typed out here."""
    script = Script(GOLDEN)
    driver = make_driver(oracle, script.config)
    replay(oracle, script, driver)
    M, T, B, p = 4, 3, 4.0, 1.0
    sizes = [10, 14, 14, 21, 29, 30]  # entries in the tree at each search, from the tree lines of the file
    pol = [r for r in driver.log if r[0] == "policy"]
    assert len(pol) == len(sizes)
    for (_, t, k, (w, s, r, z), d), n in zip(pol, sizes):
        L = 1
        while M * T ** L < n:
            L += 1
        cost = {K: w * T * L / (B * K) + s * (K * L + d / B) + r * (K * L * p + 1) + z * K * L * p for K in (1, 2)}
        assert t == 3 and k == min(cost, key=lambda K: (cost[K], K))


def test_planted_mistakes_are_noticed(oracle):
    """Variants of the driver with one rule changed must disagree with the hand-worked trace."""
    from oracle import lsm_driver_oracle as drv
    script = Script(GOLDEN)

    class EagerK(drv.DriverOracle):          # K applied to every level at once instead of on arrival
        def _observe(self, *a):
            super()._observe(*a)
            for lv in self.levels:
                lv.K = self.target_K

    class NeverAdopts(drv.DriverOracle):     # levels keep the parameters they were created with
        def flush(self, run):
            keep = (self.target_T, self.target_K)
            self.target_T, self.target_K = (self.levels[0].T, self.levels[0].K) if self.levels else keep
            super().flush(run)
            self.target_T, self.target_K = keep

    class GrowingWindow(drv.DriverOracle):   # nothing ever leaves the window
        def _slide(self):
            return sum(b[0] + b[1] + b[2] for b in self.batches)

    class DropsTombstonesEarly(drv.DriverOracle):
        def flush(self, run):
            real = drv._o.compact
            drv._o.compact = lambda runs, flags: real(runs, 1)
            try:
                super().flush(run)
            finally:
                drv._o.compact = real

    for cls in (EagerK, NeverAdopts, GrowingWindow, DropsTombstonesEarly):
        cfg = script.config
        d = cls(buffer_entries=int(cfg["M"]), T=3, K=1, window_ops=8, threshold=0.2, t_grid=(3, 3), page_entries=4.0, fpr=1.0)
        assert replay(oracle, script, d, check=False), cls.__name__
    # a wrong threshold or window length changes the policy lines as well
    assert replay(oracle, script, make_driver(oracle, script.config, threshold=0.25), check=False)
    assert replay(oracle, script, make_driver(oracle, script.config, window_ops=9), check=False)


def test_size_ratio_is_adopted_level_by_level(oracle):
    """Appendix C: a new size ratio takes effect where data flows.  With the target forced from T = 3 to T = 2 after the
    first flushes, level 1 works with capacity 4 * 2 = 8 from its next arrival on, while level 2 keeps 4 * 3**2 = 36
    until a run is moved into it and has 4 * 2**2 = 16 afterwards."""
    from oracle import lsm_driver_oracle as drv
    targets = iter([(2, 1)])
    d = drv.DriverOracle(buffer_entries=4, T=3, K=1, window_ops=4, threshold=0.2, t_grid=(2, 3), page_entries=4.0, fpr=1.0,
                         choose=lambda *a: next(targets))
    seq = [0]

    def run_of(keys):
        raw = []
        for k in keys:
            seq[0] += 1
            raw.append(brute.pack_entry(key_of(k), seq[0], brute.PUT, vptr=seq[0], vlen=1))
        return brute.run_from_raw(sorted(raw, key=lambda e: e[:32]))

    for i in range(4):                      # 16 entries: level 1 (capacity 12 at T = 3) overflows at the 4th flush
        d.flush(run_of(range(100 * i, 100 * i + 4)))
    assert [len(lv.runs) for lv in d.levels] == [0, 1] and d.levels[1].runs[0].shape[0] == 16
    assert (d.levels[0].T, d.levels[1].T) == (3, 3)
    d.writes(4)                             # window full -> the (forced) search answers T = 2
    assert d.log[-1][:3] == ("policy", 2, 1)
    assert (d.levels[0].T, d.levels[1].T) == (3, 3)         # nothing changes until data flows
    d.flush(run_of(range(400, 404)))
    assert (d.levels[0].T, d.levels[1].T) == (2, 3) and ("adopt", 1, 2, 1) in d.log
    d.flush(run_of(range(500, 504)))        # 8 entries: not more than 4 * 2, stays
    assert d.levels[0].runs[0].shape[0] == 8
    d.flush(run_of(range(600, 604)))        # 12 > 8 -> moves down; level 2 takes T = 2: 16 + 12 = 28 > 16 -> level 3
    assert ("adopt", 2, 2, 1) in d.log and d.log[-1] == ("move", 2, 3, 28)
    assert [len(lv.runs) for lv in d.levels] == [0, 0, 1] and d.levels[1].T == 2


def test_window_slides_and_threshold_holds(oracle):
    from oracle import lsm_driver_oracle as drv
    calls = []

    def choose(*a):
        calls.append(a)
        return 10, 1

    d = drv.DriverOracle(buffer_entries=100, window_ops=100, threshold=0.2, choose=choose)
    for _ in range(9):
        d.writes(10)
    assert not calls                          # 90 operations: the window is not full
    d.writes(10)
    assert len(calls) == 1 and calls[0][:4] == (1.0, 0.0, 0.0, 0.0)
    d.observe_reads(5, 4, 50)                 # 9 % reads: moved by 0.18 in L1 distance -> below the threshold
    assert len(calls) == 1
    d.observe_reads(2, 1, 20)                 # 3 + 9 + 9 x 10 = 102 >= 100: the oldest write batch leaves the window
    assert len(d.batches) == 11 and sum(b[0] for b in d.batches) == 90
    # mix (90, 7/2, 7/2, 5) / 102: moved by 12/102 + 7/102 + 5/102 = 0.235 -> a second search, with d = 70 blocks / 7 requests
    assert len(calls) == 2
    assert math.isclose(calls[1][0], 90 / 102) and math.isclose(calls[1][1], 3.5 / 102) and math.isclose(calls[1][3], 5 / 102)
    assert math.isclose(calls[1][10], 10.0)


def test_bloom_fpr_closed_forms():
    from oracle import lsm_driver_oracle as drv
    assert drv.bloom_fpr(0) == 1.0
    # one bit per key set in a huge block: the classic (1 - e^{-1/b}) of a one-hash Bloom filter with b bits per key
    for b in (4, 8, 16):
        assert math.isclose(drv.bloom_fpr(b, block_bits=1 << 16, bits_set=1), 1 - math.exp(-1 / b), rel_tol=2e-3)
    p16 = drv.bloom_fpr(16)
    assert 0.0015 < p16 < 0.003               # what the filter measures on random keys (test_oracle_bloom)
    assert drv.bloom_fpr(8) > p16 > drv.bloom_fpr(32)
