"""Token sequences -> 16-token blocks -> 32-byte prefix-preserving keys.

The paper's index layer encodes token prefixes so that lexicographic key order agrees with
prefix order (section 3.1, "disk index layer"; section 3.2).  It does not print the
encoding, so this module fixes one (it is input data: the index kernels and the checker
both treat a key as 32 opaque bytes compared as a big-endian string):

    key(block k of a sequence) = R (8 bytes) | BE16(k) | C_k (22 bytes)

  R    64-bit digest of the sequence's first block (its "family"),
  k    0-based block number,
  C_k  leading 22 bytes of a 256-bit chaining digest over blocks 0..k.

Consequences: two sequences that agree on their first k+1 blocks produce the same key for
block k (shared prefixes collide into the same index entries); if P is a proper
block-prefix of Q then key(P) < key(Q); all keys of one family are contiguous.

A second layout, the segment ladder, trades the family digest for subtree contiguity at a coarser grain (range
lookups under a long shared prefix then touch one tight key range instead of a family's whole span):

    key(block k) = D_0 D_1 ... D_7 (8 x 3 bytes) | BE16(k) | C_k (6 bytes)

  D_i  24-bit non-zero digest of the chain state after block 32 i + 31 (the end of segment i) if k >= 32 (i + 1),
       otherwise zero.

A block-prefix still sorts before its extensions (same segment: smaller k; deeper segment: a zero where the
extension has a digest), equal block-prefixes give equal keys, and all keys below a prefix of 32 g blocks share the
first 3 g bytes: the subtree is the range [D_0..D_{g-1} 00.., D_0..D_{g-1} ff..].  Sequences are limited to 256 blocks.

A key is held as four int64 "big-endian words" W0..W3 (W0 = bytes 0..7 read as a
big-endian number, and so on), so unsigned word-by-word comparison is byte-string order.
"""
from __future__ import annotations

import torch

from . import rng

VOCAB = 32000
BLOCK = 16  # tokens per block

_IV = (0x243F6A8885A308D3, 0x13198A2E03707344, 0xA4093822299F31D0, 0x082EFA98EC4E6C89)
STREAM_POOL_TOKENS = 1
STREAM_SEQ_TOKENS = 2
STREAM_REQ_TOKENS = 3


def tokens(seed: int, stream: int, owner: torch.Tensor, block: torch.Tensor) -> torch.Tensor:
    """Token ids, uniform in [0, VOCAB): shape owner.shape + (BLOCK,).

    `owner` (sequence, pool-prefix or request number) and `block` are int64 tensors of the
    same shape; token i of that block is counter (owner * 4096 + block) * 16 + i.
    """
    base = (owner * 4096 + block) * BLOCK
    idx = base.unsqueeze(-1) + torch.arange(BLOCK, device=owner.device, dtype=torch.int64)
    return rng.below(seed, stream, idx, VOCAB)


def initial_state(n: int, device) -> torch.Tensor:
    iv = torch.tensor([rng._i64(v) for v in _IV], dtype=torch.int64, device=device)
    return iv.unsqueeze(0).repeat(n, 1)


def absorb(state: torch.Tensor, toks: torch.Tensor) -> torch.Tensor:
    """One chaining step: new 256-bit state from the old one and a block of 16 tokens.

    state: [n, 4] int64, toks: [n, 16] int64 in [0, 2**32).  Two tokens are packed per
    64-bit word; every word goes through the bijective mixer into one lane, followed by a
    cross-lane add/rotate round so each output word depends on all 16 tokens.
    """
    s = [state[:, i] for i in range(4)]
    for w in range(8):
        m = (toks[:, 2 * w] << 32) | toks[:, 2 * w + 1]
        s[w & 3] = rng.mix64(s[w & 3] ^ m)
        if w & 3 == 3:
            s[0] = s[0] + s[1]
            s[2] = s[2] + s[3]
            s[1] = rng.rotl(s[1], 17) ^ s[2]
            s[3] = rng.rotl(s[3], 41) ^ s[0]
    s[0] = rng.mix64(s[0] ^ s[3])
    s[2] = rng.mix64(s[2] ^ s[1])
    return torch.stack(s, dim=1)


def family(state_after_block0: torch.Tensor) -> torch.Tensor:
    """R: 64-bit digest of a sequence's first block, from the chain state after block 0."""
    return rng.mix64(state_after_block0[:, 0] ^ rng.rotl(state_after_block0[:, 2], 29))


def make_key(fam: torch.Tensor, k: torch.Tensor, state: torch.Tensor) -> torch.Tensor:
    """[n, 4] big-endian words: R | BE16(k) | first 22 bytes of the chain state."""
    c0, c1, c2 = state[:, 0], state[:, 1], state[:, 2]
    w0 = fam
    w1 = (k << 48) | rng.lsr(c0, 16)
    w2 = (c0 << 48) | rng.lsr(c1, 16)
    w3 = (c1 << 48) | rng.lsr(c2, 16)
    return torch.stack([w0, w1, w2, w3], dim=1)


SEGMENT_BLOCKS = 32  # blocks per segment of the ladder layout (512 tokens)


def segment_digest(state: torch.Tensor) -> torch.Tensor:
    """24-bit non-zero digest of a chain state (taken at the end of a segment)."""
    return rng.lsr(rng.mix64(state[:, 0] ^ rng.rotl(state[:, 2], 13)), 40) | 1


def make_ladder_key(ladder: torch.Tensor, k: torch.Tensor, state: torch.Tensor) -> torch.Tensor:
    """[n, 4] big-endian words of the segment-ladder layout.  ladder: [n, 8] int64, the digests of the segments that
    block k lies beyond (zero elsewhere); k: block numbers < 256; state: chain state after block k."""
    d = [ladder[:, i] for i in range(8)]
    w0 = (d[0] << 40) | (d[1] << 16) | rng.lsr(d[2], 8)
    w1 = ((d[2] & 0xFF) << 56) | (d[3] << 32) | (d[4] << 8) | rng.lsr(d[5], 16)
    w2 = ((d[5] & 0xFFFF) << 48) | (d[6] << 24) | d[7]
    w3 = (k << 48) | rng.lsr(state[:, 0], 16)
    return torch.stack([w0, w1, w2, w3], dim=1)


def chain_keys(token_blocks: torch.Tensor, layout: str = "family") -> torch.Tensor:
    """Keys of every block of `n` sequences given as tokens [n, L, 16] (L <= 256): [n, L, 4] big-endian words in the
    family layout (R | k | C_k) or the ladder layout."""
    n, length = int(token_blocks.shape[0]), int(token_blocks.shape[1])
    assert length <= 8 * SEGMENT_BLOCKS and layout in ("family", "ladder")
    dev = token_blocks.device
    state = initial_state(n, dev)
    fam = None
    ladder = torch.zeros((n, 8), dtype=torch.int64, device=dev)
    out = torch.empty((n, length, 4), dtype=torch.int64, device=dev)
    for k in range(length):
        state = absorb(state, token_blocks[:, k])
        if k == 0:
            fam = family(state)
        kk = torch.full((n,), k, dtype=torch.int64, device=dev)
        out[:, k] = make_key(fam, kk, state) if layout == "family" else make_ladder_key(ladder, kk, state)
        if (k + 1) % SEGMENT_BLOCKS == 0 and (k + 1) // SEGMENT_BLOCKS <= 8:
            ladder = ladder.clone()
            ladder[:, (k + 1) // SEGMENT_BLOCKS - 1] = segment_digest(state)
    return out


def key_bytes_words(be_words: torch.Tensor) -> torch.Tensor:
    """Big-endian words -> the int64 values whose little-endian memory image is the key."""
    return rng.bswap64(be_words)


def lexsort_keys(be_words: torch.Tensor) -> torch.Tensor:
    """Permutation that sorts [n, 4] big-endian-word keys ascending as byte strings."""
    n = be_words.shape[0]
    perm = torch.arange(n, device=be_words.device, dtype=torch.int64)
    for col in (3, 2, 1, 0):
        vals = rng.ordered(be_words[perm, col])
        _, order = torch.sort(vals, stable=True)
        perm = perm[order]
    return perm
