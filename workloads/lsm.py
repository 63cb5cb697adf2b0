"""Seeded synthetic inputs for the LSM key index: sorted runs, trees and probe batches.

This module only *generates inputs* (64-byte index entries, sorted runs, probe requests).
It contains none of the arithmetic of compaction, lookup or fence building, and both the
checker and the GPU library consume what it produces.  It runs on whichever torch device
it is given, using integer operations only, so the same call yields the same bytes on the
CPU (small test cases) and on the GPU (full-size cases).

Entry layout (64 bytes; held here as eight little-endian int64 words per entry):
  words 0..3  key[32]      prefix-preserving key, ordered as a big-endian byte string
  word  4     seqno        larger = newer
  word  5     type         low byte: 0 = PUT, 1 = TOMBSTONE; upper 7 bytes zero padding
  word  6     vptr         (file_id << 32) | offset into the tensor log; opaque here
  word  7     vlen | pad   low 32 bits = bytes of the tensor block; upper 32 bits zero

The recipe follows the serving pattern the paper describes (sections 2.1 and 3.2): token
sequences arrive, many of them start with one of a pool of shared prefixes, only blocks
that are not yet cached are inserted, cached blocks are occasionally rewritten, and
eviction removes the tail of a sequence's private suffix (leaf-first), which the index
sees as tombstones.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Tuple

import torch

from . import keys as K
from . import rng

PUT = 0
TOMBSTONE = 1
VLEN_BLOCK = 16 * 40 * 1024  # 16 tokens x 40 KB per token (GLM-4-8B, paper section 4.1)

MIN_SEQ_BLOCKS, MAX_SEQ_BLOCKS = 16, 128  # 256..2048 tokens
MIN_POOL_BLOCKS, MAX_POOL_BLOCKS = 32, 96  # 512..1536 tokens

# stream numbers of the counter-based generator (one independent sequence each)
_S_POOL_LEN, _S_SEQ_LEN, _S_SEQ_HASPFX, _S_SEQ_PID = 10, 11, 12, 13
_S_OWNER_CLASS, _S_OW_PICK, _S_TB_PICK, _S_TB_CUT = 20, 21, 22, 23
_S_MULT, _S_RUNSEL, _S_KEEP, _S_TOMB, _S_SEQNO = 30, 31, 32, 33, 34
_S_REQ_LEN, _S_REQ_KIND, _S_REQ_PID, _S_REQ_SEQ, _S_REQ_FRAC = 40, 41, 42, 43, 44


# --------------------------------------------------------------------------------------
# shared-prefix pool and sequence universe
# --------------------------------------------------------------------------------------
@dataclass
class Pool:
    n: int
    plen: torch.Tensor    # [n] blocks
    states: torch.Tensor  # [n, MAX_POOL_BLOCKS, 4] chain state after block t
    fam: torch.Tensor     # [n] family digest R


def make_pool(seed: int, n_pool: int, device) -> Pool:
    pid = torch.arange(n_pool, device=device, dtype=torch.int64)
    plen = MIN_POOL_BLOCKS + rng.below(seed, _S_POOL_LEN, pid, MAX_POOL_BLOCKS - MIN_POOL_BLOCKS + 1)
    state = K.initial_state(n_pool, device)
    states = torch.empty((n_pool, MAX_POOL_BLOCKS, 4), dtype=torch.int64, device=device)
    for t in range(MAX_POOL_BLOCKS):
        toks = K.tokens(seed, K.STREAM_POOL_TOKENS, pid, torch.full_like(pid, t))
        state = K.absorb(state, toks)
        states[:, t] = state
    return Pool(n_pool, plen, states, K.family(states[:, 0]))


@dataclass
class Universe:
    """Distinct index keys in arrival order: pool prefixes first, then each sequence's
    private suffix blocks, sequence by sequence."""
    seed: int
    pool: Pool
    zipf_a: Optional[float]
    keys: torch.Tensor        # [N, 4] big-endian words
    owner: torch.Tensor       # [N] pool id, or n_pool + sequence number
    rank: torch.Tensor        # [N] position of the key in ascending key order
    n_pool_entries: int
    seq_len: torch.Tensor     # [S] blocks
    seq_pid: torch.Tensor     # [S] pool id or -1
    seq_shared: torch.Tensor  # [S] leading blocks taken from the pool prefix
    seq_ulen: torch.Tensor    # [S] private blocks inserted by this sequence
    seq_first: torch.Tensor   # [S] arrival index of its first private block

    @property
    def n(self) -> int:
        return int(self.keys.shape[0])


def _draw_sequences(seed: int, pool: Pool, zipf_a: Optional[float], s0: int, s1: int, device):
    sid = torch.arange(s0, s1, device=device, dtype=torch.int64)
    length = MIN_SEQ_BLOCKS + rng.below(seed, _S_SEQ_LEN, sid, MAX_SEQ_BLOCKS - MIN_SEQ_BLOCKS + 1)
    has = rng.chance(seed, _S_SEQ_HASPFX, sid, 0.6)
    if zipf_a is None:
        pid = rng.below(seed, _S_SEQ_PID, sid, pool.n)
    else:
        thr = torch.from_numpy(rng.zipf_thresholds(pool.n, zipf_a)).to(device)
        pid = rng.zipf(seed, _S_SEQ_PID, sid, thr)
    shared = torch.where(has, torch.minimum(pool.plen[pid], length), torch.zeros_like(length))
    pid = torch.where(has, pid, torch.full_like(pid, -1))
    return length, pid, shared, length - shared


def make_universe(seed: int, n_entries: int, n_pool: int, zipf_a: Optional[float], device,
                  chunk: int = 1 << 20) -> Universe:
    """Exactly `n_entries` distinct keys (pool prefixes + as many sequences as needed)."""
    pool = make_pool(seed, n_pool, device)
    pool_first = torch.cumsum(pool.plen, 0) - pool.plen
    n_pool_entries = int(pool.plen.sum().item())
    assert n_entries > n_pool_entries, "entry target smaller than the shared-prefix pool"
    need = n_entries - n_pool_entries

    # draw sequences until their private blocks cover the target; the last one is cut short
    parts, got, s0 = [], 0, 0
    while got < need:
        s1 = s0 + max(1024, min(chunk, (need - got) // 30 + 1024))
        part = _draw_sequences(seed, pool, zipf_a, s0, s1, device)
        parts.append(part)
        got += int(part[3].sum().item())
        s0 = s1
    length, pid, shared, ulen = (torch.cat([p[i] for p in parts]) for i in range(4))
    csum = torch.cumsum(ulen, 0)
    n_seq = int(torch.searchsorted(csum, torch.tensor([need], device=device)).item()) + 1
    length, pid, shared, ulen = length[:n_seq].clone(), pid[:n_seq], shared[:n_seq], ulen[:n_seq].clone()
    excess = int(csum[n_seq - 1].item()) - need
    ulen[-1] -= excess
    length[-1] -= excess
    first = n_pool_entries + torch.cumsum(ulen, 0) - ulen

    keys = torch.empty((n_entries, 4), dtype=torch.int64, device=device)
    owner = torch.empty(n_entries, dtype=torch.int64, device=device)

    # pool prefixes: block t of prefix p, for t < plen[p]
    for t in range(MAX_POOL_BLOCKS):
        act = torch.nonzero(pool.plen > t).squeeze(1)
        dst = pool_first[act] + t
        keys[dst] = K.make_key(pool.fam[act], torch.full_like(act, t), pool.states[act, t])
        owner[dst] = act

    # sequences: chain continues from the pool state (or the IV) over the private blocks
    for c0 in range(0, n_seq, chunk):
        c1 = min(n_seq, c0 + chunk)
        sid = torch.arange(c0, c1, device=device, dtype=torch.int64)
        c_pid, c_sh, c_ul, c_first = pid[c0:c1], shared[c0:c1], ulen[c0:c1], first[c0:c1]
        has = c_pid >= 0
        safe_pid = c_pid.clamp(min=0)
        state = torch.where(has.unsqueeze(1), pool.states[safe_pid, (c_sh - 1).clamp(min=0)],
                            K.initial_state(c1 - c0, device))
        fam = pool.fam[safe_pid].clone()
        for u in range(int(c_ul.max().item()) if c1 > c0 else 0):
            act = torch.nonzero(c_ul > u).squeeze(1)
            blk = c_sh[act] + u
            st = K.absorb(state[act], K.tokens(seed, K.STREAM_SEQ_TOKENS, sid[act], blk))
            state[act] = st
            if u == 0:
                own = ~has[act]
                fam[act[own]] = K.family(st[own])
            dst = c_first[act] + u
            keys[dst] = K.make_key(fam[act], blk, st)
            owner[dst] = n_pool + sid[act]

    order = K.lexsort_keys(keys)
    sk = keys[order]
    if n_entries > 1:
        assert bool((sk[1:] != sk[:-1]).any(dim=1).all().item()), "key digest collision in universe"
    rank = torch.empty(n_entries, dtype=torch.int64, device=device)
    rank[order] = torch.arange(n_entries, device=device, dtype=torch.int64)
    return Universe(seed, pool, zipf_a, keys, owner, rank, n_pool_entries,
                    length, pid, shared, ulen, first)


# --------------------------------------------------------------------------------------
# entries and runs
# --------------------------------------------------------------------------------------
def _assemble(U: Universe, idx: torch.Tensor, seqno: torch.Tensor, typ: torch.Tensor,
              group: Optional[torch.Tensor] = None) -> torch.Tensor:
    """[n, 8] int64 entries for universe indices `idx`, sorted ascending by key (within each
    `group` number, groups in ascending order, if given)."""
    sort_key = U.rank[idx] if group is None else group * (1 << 40) + U.rank[idx]
    order = torch.argsort(sort_key)
    idx, seqno, typ = idx[order], seqno[order], typ[order]
    e = torch.empty((idx.numel(), 8), dtype=torch.int64, device=idx.device)
    e[:, 0:4] = K.key_bytes_words(U.keys[idx])
    e[:, 4] = seqno
    e[:, 5] = typ
    put = typ == PUT
    file_id, offset = rng.lsr(seqno, 12) & 0xFFFFFFFF, seqno & 0xFFF
    e[:, 6] = torch.where(put, (file_id << 32) | offset, torch.zeros_like(seqno))
    e[:, 7] = torch.where(put, torch.full_like(seqno, VLEN_BLOCK), torch.zeros_like(seqno))
    return e


def _pick_smallest_hash(seed: int, stream: int, cand: torch.Tensor, m: int) -> torch.Tensor:
    """`m` distinct elements of `cand`: those with the smallest per-element hash."""
    assert m <= cand.numel()
    if m == 0:
        return cand[:0]
    h = rng.lsr(rng.u64(seed, stream, cand), 1)
    if cand.numel() > 4 * m + 4096:  # thin out before sorting
        thr = int(min(1.0, 1.5 * m / cand.numel() + 1e-4) * (1 << 63))
        keep = h < thr
        if int(keep.sum().item()) >= m:
            cand, h = cand[keep], h[keep]
    # ties on the 63-bit hash are broken by the element itself
    order = torch.argsort(cand)
    cand, h = cand[order], h[order]
    return cand[torch.sort(h, stable=True)[1][:m]]


def _tomb_eligible(U: Universe, owner: torch.Tensor) -> torch.Tensor:
    """Sequences whose private tail may be evicted (a fixed quarter of them; never the pool)."""
    return (owner >= U.pool.n) & ((rng.u64(U.seed, _S_OWNER_CLASS, owner) & 3) == 0)


def epoch_runs(U: Universe, sizes_old_to_new: List[int], ow_frac: float, tb_frac: float) -> List[torch.Tensor]:
    """Cut one operation stream into runs (epochs).  Returns runs NEWEST FIRST (see epoch_runs_state)."""
    return epoch_runs_state(U, sizes_old_to_new, ow_frac, tb_frac)[0]


def epoch_runs_state(U: Universe, sizes_old_to_new: List[int], ow_frac: float, tb_frac: float):
    """Cut one operation stream into runs (epochs).  Returns (runs NEWEST FIRST, number of universe
    entries consumed as fresh inserts, next unused seqno).

    Epoch 0 (oldest) holds fresh inserts only.  Every later epoch of n entries holds
    round(n*ow_frac) overwrites (a new PUT, newer seqno and pointer, for a key inserted in
    an older epoch), about round(n*tb_frac) tombstones (the tail of the private suffix of a
    sequence inserted in older epochs) and fresh inserts for the rest.  Keys are distinct
    within an epoch, seqnos increase with time, so a newer run always holds the newer
    version of a shared key.
    """
    dev = U.keys.device
    n_epochs = len(sizes_old_to_new)
    runs, fp, base = [], 0, 0
    seq_owner = U.pool.n + torch.arange(U.seq_ulen.numel(), device=dev, dtype=torch.int64)
    seq_elig = _tomb_eligible(U, seq_owner) & (U.seq_ulen > 0)
    seq_epoch = (rng.lsr(rng.u64(U.seed, _S_OWNER_CLASS, seq_owner), 2) % max(1, n_epochs - 1)) + 1
    seq_end = U.seq_first + U.seq_ulen
    for e, n_e in enumerate(sizes_old_to_new):
        if e == 0:
            n_ow = n_tb = 0
            tb_idx = ow_idx = torch.empty(0, dtype=torch.int64, device=dev)
        else:
            n_ow, n_tb = int(round(n_e * ow_frac)), int(round(n_e * tb_frac))
            tb_idx = torch.empty(0, dtype=torch.int64, device=dev)
            # tombstones: tails of victim sequences that were fully inserted before this epoch
            vict = torch.nonzero(seq_elig & (seq_epoch == e) & (seq_end <= fp)).squeeze(1)
            vict = _pick_smallest_hash(U.seed, _S_TB_PICK + 100 * e, vict, vict.numel())
            cut = rng.lsr(rng.u64(U.seed, _S_TB_CUT, vict), 33) % U.seq_ulen[vict]
            tail = U.seq_ulen[vict] - cut
            csum = torch.cumsum(tail, 0)
            n_tb = min(n_tb, int(csum[-1].item()) if vict.numel() else 0)
            if n_tb > 0:
                nv = int(torch.searchsorted(csum, torch.tensor([n_tb], device=dev)).item()) + 1
                vict, tail, cut = vict[:nv], tail[:nv].clone(), cut[:nv].clone()
                over = int(csum[nv - 1].item()) - n_tb
                tail[-1] -= over
                cut[-1] += over
                start = U.seq_first[vict] + cut
                rep = torch.repeat_interleave(torch.arange(nv, device=dev), tail)
                within = torch.arange(n_tb, device=dev) - (torch.cumsum(tail, 0) - tail)[rep]
                tb_idx = start[rep] + within
            # overwrites: older keys of owners that are never evicted
            older = torch.arange(fp, device=dev, dtype=torch.int64)
            cand = older[~_tomb_eligible(U, U.owner[:fp])]
            n_ow = min(n_ow, cand.numel())
            ow_idx = _pick_smallest_hash(U.seed, _S_OW_PICK + 100 * e, cand, n_ow)
        n_fresh = n_e - n_ow - n_tb
        assert fp + n_fresh <= U.n, "universe too small for the requested runs"
        fresh_idx = torch.arange(fp, fp + n_fresh, device=dev, dtype=torch.int64)
        idx = torch.cat([fresh_idx, ow_idx, tb_idx])
        seqno = base + torch.arange(n_e, device=dev, dtype=torch.int64)
        typ = torch.cat([torch.zeros(n_fresh + n_ow, dtype=torch.int64, device=dev),
                         torch.ones(n_tb, dtype=torch.int64, device=dev)])
        runs.append(_assemble(U, idx, seqno, typ))
        fp += n_fresh
        base += n_e
    return runs[::-1], fp, base


def fresh_needed(sizes_old_to_new: List[int], ow_frac: float, tb_frac: float) -> int:
    """Upper bound on distinct keys `epoch_runs` consumes (tombstones may fall short)."""
    return sizes_old_to_new[0] + sum(n - int(round(n * ow_frac)) for n in sizes_old_to_new[1:])


def overlapping_runs(U: Universe, n_runs: int, run_len: int, dup_frac: float, tb_frac: float) -> List[torch.Tensor]:
    """Tiered-compaction input: `n_runs` runs of exactly `run_len` entries over one key set.

    A fraction `dup_frac` of the distinct keys appears in m runs, m uniform in {2,3,4}, the
    others in one; runs are chosen uniformly; seqnos are unique and random (a bijective mix
    of the instance number, full 64-bit range); `tb_frac` of the instances are tombstones.
    Surplus instances of a run (lowest keep-hash first kept) are dropped to hit `run_len`.
    """
    dev, seed = U.keys.device, U.seed
    u = torch.arange(U.n, device=dev, dtype=torch.int64)
    dup = rng.chance(seed, _S_MULT, u, dup_frac)
    mult = torch.where(dup, 2 + rng.below(seed, _S_MULT + 1, u, 3), torch.ones_like(u))
    r0 = rng.below(seed, _S_RUNSEL, u, n_runs)
    step = 2 * rng.below(seed, _S_RUNSEL + 1, u, max(1, n_runs // 2)) + 1  # odd: distinct runs
    rep = torch.repeat_interleave(u, mult)
    j = torch.arange(rep.numel(), device=dev, dtype=torch.int64) - (torch.cumsum(mult, 0) - mult)[rep]
    run = (r0[rep] + j * step[rep]) % n_runs
    inst = torch.arange(rep.numel(), device=dev, dtype=torch.int64)
    seqno = rng.mix64(inst ^ rng.stream_key(seed, _S_SEQNO))
    typ = rng.chance(seed, _S_TOMB, inst, tb_frac).to(torch.int64)
    keep_hash = rng.lsr(rng.u64(seed, _S_KEEP, inst), 1)
    runs = []
    for r in range(n_runs):
        sel = torch.nonzero(run == r).squeeze(1)
        assert sel.numel() >= run_len, f"run {r}: {sel.numel()} candidates < {run_len}"
        sel = sel[torch.sort(keep_hash[sel], stable=True)[1][:run_len]]
        runs.append(_assemble(U, rep[sel], seqno[sel], typ[sel]))
    return runs


# --------------------------------------------------------------------------------------
# probe requests
# --------------------------------------------------------------------------------------
def make_queries(U: Universe, n_req: int, min_blocks: int, max_blocks: int, p_pool: float, p_plain: float,
                 zipf_a: Optional[float], stream: int = 0, row_blocks: Optional[int] = None
                 ) -> Tuple[torch.Tensor, torch.Tensor]:
    """A batch of longest-prefix probe requests.

    Returns (keys, n_blocks): keys is [n_req, row_blocks, 4] int64 whose memory image is
    row_blocks x 32 key bytes per request (zero beyond n_blocks), n_blocks is int32 [n_req].
    With probability p_pool a request follows a stored sequence that starts with a pool
    prefix (prefix chosen uniformly or Zipf), with probability p_plain one without a pool
    prefix; it follows that sequence's private blocks for a random fraction and continues
    with tokens of its own.  Otherwise every token is its own (a miss at block 0).
    """
    dev, seed, pool = U.keys.device, U.seed, U.pool
    row_blocks = row_blocks or max_blocks
    rid = (stream << 32) + torch.arange(n_req, device=dev, dtype=torch.int64)
    nb = min_blocks + rng.below(seed, _S_REQ_LEN, rid, max_blocks - min_blocks + 1)
    kind_r = rng.lsr(rng.u64(seed, _S_REQ_KIND, rid), 33)
    t_pool, t_plain = int(p_pool * (1 << 31)), int((p_pool + p_plain) * (1 << 31))
    want_pool, want_plain = kind_r < t_pool, (kind_r >= t_pool) & (kind_r < t_plain)

    # sequences grouped by pool id (group -1 = no pool prefix), for "pick one with this prefix"
    n_seq = U.seq_pid.numel()
    order = torch.sort(U.seq_pid, stable=True)[1]
    counts = torch.bincount(U.seq_pid + 1, minlength=pool.n + 1)
    gfirst = torch.cumsum(counts, 0) - counts
    if zipf_a is None:
        pid = rng.below(seed, _S_REQ_PID, rid, pool.n)
    else:
        thr = torch.from_numpy(rng.zipf_thresholds(pool.n, zipf_a)).to(dev)
        pid = rng.zipf(seed, _S_REQ_PID, rid, thr)
    group = torch.where(want_pool, pid + 1, torch.zeros_like(pid))
    gcount = counts[group]
    pick = rng.lsr(rng.u64(seed, _S_REQ_SEQ, rid), 1) % gcount.clamp(min=1)
    follows = (want_pool | want_plain) & (gcount > 0) & (n_seq > 0)
    seq = torch.where(follows, order[(gfirst[group] + pick).clamp(max=max(n_seq - 1, 0))], torch.zeros_like(pid))
    # a request that wanted a pool prefix no stored sequence uses still carries that prefix
    pool_only = want_pool & ~follows
    shared = torch.where(follows, U.seq_shared[seq], torch.where(pool_only, pool.plen[pid], torch.zeros_like(pid)))
    src_pid = torch.where(follows, U.seq_pid[seq], torch.where(pool_only, pid, torch.full_like(pid, -1))).clamp(min=0)
    frac = rng.below(seed, _S_REQ_FRAC, rid, 257)
    follow_u = torch.where(follows, (U.seq_ulen[seq] * frac) >> 8, torch.zeros_like(pid))

    keys = torch.zeros((n_req, row_blocks, 4), dtype=torch.int64, device=dev)
    state = K.initial_state(n_req, dev)
    fam = torch.zeros(n_req, dtype=torch.int64, device=dev)
    for t in range(int(nb.max().item()) if n_req else 0):
        act = torch.nonzero(nb > t).squeeze(1)
        tt = torch.full_like(act, t)
        in_pool = t < shared[act]
        in_seq = ~in_pool & (t < shared[act] + follow_u[act])
        toks = K.tokens(seed, K.STREAM_REQ_TOKENS, rid[act], tt)
        toks = torch.where(in_seq.unsqueeze(1), K.tokens(seed, K.STREAM_SEQ_TOKENS, seq[act], tt), toks)
        toks = torch.where(in_pool.unsqueeze(1), K.tokens(seed, K.STREAM_POOL_TOKENS, src_pid[act], tt), toks)
        st = K.absorb(state[act], toks)
        state[act] = st
        if t == 0:
            fam[act] = K.family(st)
        keys[act, t] = K.key_bytes_words(K.make_key(fam[act], tt, st))
    return keys, nb.to(torch.int32)


# --------------------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    universe: Universe
    runs: List[torch.Tensor]          # newest first; each [n, 8] int64
    levels: List[int]                 # tree level of each run (1 = shallowest)
    bottommost: bool                  # whether the compaction of `runs` targets the last level


def config1(device="cpu", seed: int = rng.SEED) -> Workload:
    """L0->L1: 4 overlapping runs of 16,384 entries cut from one operation stream."""
    sizes = [16384] * 4
    ow, tb = 0.10 * 4 / 3, 0.05 * 4 / 3  # 10 % / 5 % of all entries, carried by the 3 newer runs
    U = make_universe(seed, fresh_needed(sizes, ow, tb) + 1, 64, None, device)
    return Workload("cfg1_l0_l1_4x16k", U, epoch_runs(U, sizes, ow, tb), [0, 0, 0, 0], False)


def config2(device="cpu", seed: int = rng.SEED, scale: int = 1) -> Workload:
    """Leveled L1->L2, size ratio 10: a 2M-entry run (newer) merged into a 20M-entry run."""
    sizes = [20_000_000 // scale, 2_000_000 // scale]
    n_pool = max(16, 4096 // scale)
    U = make_universe(seed + 2, fresh_needed(sizes, 0.08, 0.03) + 1, n_pool, 0.9, device)
    return Workload(f"cfg2_leveled_2m_20m_div{scale}", U, epoch_runs(U, sizes, 0.08, 0.03), [1, 2], False)


def config3(device="cpu", seed: int = rng.SEED, scale: int = 1) -> Workload:
    """Tiered 16-way merge into the last level: 16 runs x 4,194,304 entries."""
    n_runs, run_len = 16, 4_194_304 // scale
    n_pool = max(16, 4096 // scale)
    # expected instances per key = 0.8 + 0.2 * 3 = 1.4; 3 % surplus so every run can be cut to size
    n_keys = int(n_runs * run_len / 1.4 * 1.03) + 4096
    U = make_universe(seed + 3, n_keys, n_pool, 0.9, device)
    return Workload(f"cfg3_tiered_16x4m_div{scale}", U, overlapping_runs(U, n_runs, run_len, 0.20, 0.05),
                    [1] * n_runs, True)


def tree_sizes(total: int, n_levels: int, ratio: int) -> List[int]:
    """Level sizes proportional to ratio**(i-1), the remainder going to the last level."""
    denom = sum(ratio ** i for i in range(n_levels))
    sizes = [total * ratio ** i // denom for i in range(n_levels - 1)]
    return sizes + [total - sum(sizes)]


def config4(device="cpu", seed: int = rng.SEED, scale: int = 1) -> Workload:
    """Lookup-heavy: a 5-level leveled tree of 100M entries, size ratio 10."""
    sizes = tree_sizes(100_000_000 // scale, 5, 10)  # shallow -> deep
    n_pool = max(16, 4096 // scale)
    old_to_new = sizes[::-1]
    U = make_universe(seed + 4, fresh_needed(old_to_new, 0.08, 0.03) + 1, n_pool, 0.9, device)
    return Workload(f"cfg4_tree5_100m_div{scale}", U, epoch_runs(U, old_to_new, 0.08, 0.03), [1, 2, 3, 4, 5], False)


def config5_tree(device="cpu", seed: int = rng.SEED, scale: int = 1) -> Workload:
    """Starting tree of the mixed workload: 6 levels, 400M entries, size ratio 10."""
    sizes = tree_sizes(400_000_000 // scale, 6, 10)
    n_pool = max(16, 4096 // scale)
    old_to_new = sizes[::-1]
    U = make_universe(seed + 5, fresh_needed(old_to_new, 0.08, 0.05) + 1, n_pool, 0.9, device)
    return Workload(f"cfg5_tree6_400m_div{scale}", U, epoch_runs(U, old_to_new, 0.08, 0.05), [1, 2, 3, 4, 5, 6], False)


def queries_config1(w: Workload, n_req: int = 4096, stream: int = 0):
    return make_queries(w.universe, n_req, MIN_SEQ_BLOCKS, MAX_SEQ_BLOCKS, 0.60, 0.25, None, stream, row_blocks=256)


def queries_config4(w: Workload, n_req: int = 4096, stream: int = 0):
    """Zipf(0.99) over the prefix pool, 30 % misses, 16..256 blocks per request."""
    return make_queries(w.universe, n_req, 16, 256, 0.70, 0.0, 0.99, stream, row_blocks=256)


# --------------------------------------------------------------------------------------
# configuration 5: mixed, shifting workload on a leveled tree
# --------------------------------------------------------------------------------------
@dataclass
class MixedTrace:
    """Starting tree plus a time-ordered trace of flushes (sorted runs of `buffer_entries`
    entries from the write buffer) and probe batches."""
    workload: Workload                 # starting tree, runs newest first, one per level
    buffer_entries: int                # M: entries per flushed run
    size_ratio: int                    # T of the starting tree
    flush_runs: torch.Tensor           # [n_flushes, M, 8]
    events: List[Tuple[str, int, int]]  # ("flush", f, phase) / ("probe", b, phase) in time order
    batch_requests: int
    write_ops_between: List[int]       # write operations (sequences) that happened before each event since the last one

    def probe_batch(self, b: int):
        return make_queries(self.workload.universe, self.batch_requests, 16, 256, 0.70, 0.0, 0.99, stream=1000 + b,
                            row_blocks=256)


_S_OP_KIND, _S_FLUSH_TB, _S_FLUSH_CUT = 50, 51, 52


def config5(device="cpu", seed: int = rng.SEED, tree_total: int = 400_000_000, buffer_entries: int = 3600,
            ops_per_phase: int = 1 << 18, batch_requests: int = 4096, tb_frac: float = 0.05,
            read_shares=(0.9, 0.5, 0.1)) -> MixedTrace:
    """Mixed workload: a leveled tree (size ratio 10, level i holds M * 10**(i-1) entries, the last
    level the remainder) and three phases of `ops_per_phase` operations with read shares
    90 %, 50 %, 10 %.  A read is one probe request (batches of `batch_requests`); a write inserts
    the not-yet-present blocks of the next sequence into the write buffer, which is flushed as a
    sorted run every `buffer_entries` entries, `tb_frac` of them tombstones for tails of
    sequences of the starting tree."""
    T = 10
    n_levels = 1
    while buffer_entries * T ** n_levels < tree_total:
        n_levels += 1
    sizes = tree_sizes(tree_total, n_levels, T)
    old_to_new = sizes[::-1]
    n_ops = 3 * ops_per_phase
    n_write_est = int(sum((1 - r) * ops_per_phase for r in read_shares))
    n_pool = max(16, min(4096, tree_total // 100_000))
    U = make_universe(seed + 5, fresh_needed(old_to_new, 0.08, tb_frac) + 45 * n_write_est + 4096, n_pool, 0.9, device)
    runs, fp, next_seq = epoch_runs_state(U, old_to_new, 0.08, tb_frac)
    w = Workload(f"cfg5_tree{n_levels}_{tree_total}", U, runs, list(range(1, n_levels + 1)), False)
    dev = U.keys.device

    # operations: write or read, by phase
    op = torch.arange(n_ops, device=dev, dtype=torch.int64)
    phase = op // ops_per_phase
    thr = torch.tensor([int((1 - r) * (1 << 31)) for r in read_shares], device=dev, dtype=torch.int64)
    is_write = rng.lsr(rng.u64(seed, _S_OP_KIND, op), 33) < thr[phase]
    n_writes_before = torch.cumsum(is_write.to(torch.int64), 0)   # inclusive
    n_reads_before = torch.cumsum((~is_write).to(torch.int64), 0)
    # write k inserts the private blocks of the k-th sequence after the ones the tree used up
    seq_end = U.seq_first + U.seq_ulen
    s0 = int(torch.searchsorted(seq_end, torch.tensor([fp], device=dev), right=True).item())  # first sequence with blocks >= fp
    n_seq_avail = U.seq_ulen.numel() - s0
    seq_of_write = s0 + torch.arange(min(int(n_writes_before[-1].item()), n_seq_avail), device=dev)
    ends = torch.clamp(seq_end[seq_of_write], min=fp) - fp        # fresh entries written after each write op
    m_tb = int(round(buffer_entries * tb_frac))
    m_fresh = buffer_entries - m_tb
    n_flushes = int(ends[-1].item()) // m_fresh if ends.numel() else 0
    # event times: flush f right after the write that fills the buffer, probe batch b after its last read
    write_pos = torch.nonzero(is_write).squeeze(1)[: ends.numel()]
    fl_targets = (torch.arange(n_flushes, device=dev, dtype=torch.int64) + 1) * m_fresh
    fl_write = torch.searchsorted(ends, fl_targets)               # index of the write op that reaches the target
    fl_op = write_pos[fl_write]
    n_batches = int(n_reads_before[-1].item()) // batch_requests
    pb_targets = (torch.arange(n_batches, device=dev, dtype=torch.int64) + 1) * batch_requests
    pb_op = torch.searchsorted(n_reads_before, pb_targets)
    ev = [("flush", f, int(o)) for f, o in enumerate(fl_op.tolist())] + [("probe", b, int(o)) for b, o in enumerate(pb_op.tolist())]
    ev.sort(key=lambda e: (e[2], 0 if e[0] == "flush" else 1))
    events, writes_between, last_w = [], [], 0
    nwb = n_writes_before.cpu()
    for kind, i, o in ev:
        events.append((kind, i, o // ops_per_phase))
        wb = int(nwb[o])
        writes_between.append(wb - last_w)
        last_w = wb

    # flushed runs: fresh slice + tombstones for tails of tree sequences, sorted per flush
    if n_flushes:
        fresh_idx = fp + torch.arange(n_flushes * m_fresh, device=dev, dtype=torch.int64)
        fresh_flush = torch.arange(n_flushes * m_fresh, device=dev, dtype=torch.int64) // m_fresh
        seq_owner = U.pool.n + torch.arange(U.seq_ulen.numel(), device=dev, dtype=torch.int64)
        vict = torch.nonzero(_tomb_eligible(U, seq_owner) & (U.seq_ulen > 0) & (seq_end <= fp)).squeeze(1)
        vict = _pick_smallest_hash(seed, _S_FLUSH_TB, vict, vict.numel())
        cut = rng.lsr(rng.u64(seed, _S_FLUSH_CUT, vict), 33) % U.seq_ulen[vict]
        tail = U.seq_ulen[vict] - cut
        need_tb = n_flushes * m_tb
        csum = torch.cumsum(tail, 0)
        assert vict.numel() and int(csum[-1].item()) >= need_tb, "not enough evictable tails for the trace"
        nv = int(torch.searchsorted(csum, torch.tensor([need_tb], device=dev)).item()) + 1
        vict, tail, cut = vict[:nv], tail[:nv].clone(), cut[:nv].clone()
        over = int(csum[nv - 1].item()) - need_tb
        tail[-1] -= over
        cut[-1] += over
        rep_ = torch.repeat_interleave(torch.arange(nv, device=dev), tail)
        within = torch.arange(need_tb, device=dev) - (torch.cumsum(tail, 0) - tail)[rep_]
        tb_idx = (U.seq_first[vict] + cut)[rep_] + within
        tb_flush = torch.arange(need_tb, device=dev, dtype=torch.int64) // max(m_tb, 1)
        idx = torch.cat([fresh_idx, tb_idx])
        flush_id = torch.cat([fresh_flush, tb_flush])
        within_flush = torch.cat([torch.arange(n_flushes * m_fresh, device=dev) % m_fresh,
                                  m_fresh + torch.arange(need_tb, device=dev) % max(m_tb, 1)])
        seqno = next_seq + flush_id * buffer_entries + within_flush
        typ = torch.cat([torch.zeros(n_flushes * m_fresh, dtype=torch.int64, device=dev),
                         torch.ones(need_tb, dtype=torch.int64, device=dev)])
        flush_runs = _assemble(U, idx, seqno, typ, group=flush_id).view(n_flushes, buffer_entries, 8)
    else:
        flush_runs = torch.empty((0, buffer_entries, 8), dtype=torch.int64, device=dev)
    return MixedTrace(w, buffer_entries, T, flush_runs, events, batch_requests, writes_between)
