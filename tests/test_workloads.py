"""Properties of the seeded input generator (CPU only)."""
import numpy as np
import pytest
import torch

from workloads import keys as K
from workloads import lsm, rng


def _key_bytes(words):  # [n, 4] memory words -> list of 32-byte strings
    a = words.contiguous().numpy().view(np.uint8).reshape(-1, 32)
    return [a[i].tobytes() for i in range(a.shape[0])]


def test_mixer_is_the_published_splitmix64():
    # first outputs of splitmix64 seeded with 0 (state advances by the golden-ratio increment)
    want = [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]
    state, got = 0, []
    for _ in range(3):
        got.append(rng.mix64_int(state))
        state = (state + 0x9E3779B97F4A7C15) & ((1 << 64) - 1)
    assert got == want
    x = torch.tensor([0, rng._i64(0x9E3779B97F4A7C15)], dtype=torch.int64)
    assert [int(v) & ((1 << 64) - 1) for v in rng.mix64(x)] == want[:2]


def test_bswap_and_order_helpers():
    x = torch.tensor([0x0102030405060708, -2], dtype=torch.int64)
    assert int(rng.bswap64(x)[0]) == 0x0807060504030201
    assert int(rng.bswap64(rng.bswap64(x))[1]) == -2
    v = torch.tensor([0, 1, (1 << 63) - 1, -(1 << 63), -1], dtype=torch.int64)  # unsigned ascending
    o = rng.ordered(v)
    assert bool((o[1:] > o[:-1]).all())


def test_keys_preserve_prefix_order():
    """A block-prefix sorts before its extensions; equal block-prefixes give equal keys."""
    w = lsm.config1()
    U = w.universe
    q, nb = lsm.make_queries(U, 64, 16, 64, 0.6, 0.4, None, stream=3, row_blocks=64)
    for i in range(64):
        ks = _key_bytes(q[i, : int(nb[i])])
        assert all(ks[j] < ks[j + 1] for j in range(len(ks) - 1))
        assert len({k[:8] for k in ks}) == 1  # one family
        assert [int.from_bytes(k[8:10], "big") for k in ks] == list(range(len(ks)))
    # two requests following the same stored sequence share keys exactly as far as they share tokens
    q2, nb2 = lsm.make_queries(U, 64, 16, 64, 0.6, 0.4, None, stream=3, row_blocks=64)
    assert torch.equal(q, q2) and torch.equal(nb, nb2)


def test_runs_are_strictly_sorted_and_sized():
    for w, sizes in ((lsm.config1(), [16384] * 4), (lsm.config3(scale=1024), [4096] * 16),
                     (lsm.config2(scale=500), [4000, 40000]), (lsm.config4(scale=1000), None)):
        if sizes:
            assert [int(r.shape[0]) for r in w.runs] == sizes
        for r in w.runs:
            ks = _key_bytes(r[:, 0:4])
            assert all(ks[j] < ks[j + 1] for j in range(len(ks) - 1))
            assert set(r[:, 5].tolist()) <= {0, 1}
            tomb = r[:, 5] == 1
            assert bool((r[tomb][:, 6:8] == 0).all()) and bool((r[~tomb][:, 7] == lsm.VLEN_BLOCK).all())


def test_config_fractions():
    w = lsm.config1()
    allk = torch.cat([r[:, 0:4] for r in w.runs])
    n_dist = torch.unique(allk, dim=0).shape[0]
    tomb = sum(int((r[:, 5] == 1).sum()) for r in w.runs) / allk.shape[0]
    assert 0.12 < 1 - n_dist / allk.shape[0] < 0.16 and 0.035 < tomb < 0.055
    w = lsm.config3(scale=256)
    allk = torch.cat([r[:, 0:4] for r in w.runs])
    n_dist = torch.unique(allk, dim=0).shape[0]
    assert 0.70 < n_dist / allk.shape[0] < 0.74  # 1 / 1.4
    tomb = sum(int((r[:, 5] == 1).sum()) for r in w.runs) / allk.shape[0]
    assert 0.045 < tomb < 0.055
    seq = torch.cat([r[:, 4] for r in w.runs])
    assert torch.unique(seq).numel() == seq.numel() and int((seq < 0).sum()) > seq.numel() // 3  # full 64-bit range


def test_tree_sizes():
    assert lsm.tree_sizes(100_000_000, 5, 10) == [9000, 90000, 900009, 9000090, 90000901]
    s = lsm.tree_sizes(400_000_000, 6, 10)
    assert s[0] == 3600 and sum(s) == 400_000_000 and s[-1] > 360_000_000


def test_generator_is_deterministic():
    a, b = lsm.config3(scale=2048), lsm.config3(scale=2048)
    assert all(torch.equal(x, y) for x, y in zip(a.runs, b.runs))


def _prefix_tree_tokens(n_seq=60, length=100, seed=9):
    """Sequences that share prefixes of many lengths: sequence i copies the first cut[i] blocks of an earlier one."""
    import numpy as np
    rs = np.random.RandomState(seed)
    toks = rs.randint(0, 32000, size=(n_seq, length, 16)).astype(np.int64)
    parent, cut = [-1] * n_seq, [0] * n_seq
    for i in range(1, n_seq):
        if rs.rand() < 0.8:
            parent[i] = int(rs.randint(0, i))
            cut[i] = int(rs.choice([1, 5, 16, 31, 32, 33, 40, 64, 65, 96, 99]))
            toks[i, :cut[i]] = toks[parent[i], :cut[i]]
    return torch.from_numpy(toks)


def _as_bytes(words):
    from workloads import keys as K
    return [bytes(r) for r in K.key_bytes_words(words.reshape(-1, 4)).numpy().view("u1").reshape(-1, 32)]


@pytest.mark.parametrize("layout", ["family", "ladder"])
def test_both_key_layouts_follow_prefix_order(layout):
    """Equal block-prefixes give equal keys, different ones different keys, and a prefix sorts before its extensions."""
    from workloads import keys as K
    toks = _prefix_tree_tokens()
    n, length = toks.shape[0], toks.shape[1]
    kb = _as_bytes(K.chain_keys(toks, layout))
    key = lambda i, k: kb[i * length + k]
    for i in range(n):
        for k in range(length - 1):
            assert key(i, k) < key(i, k + 1)                       # a block-prefix before its extension
    t = toks.numpy()
    for i in range(0, n, 7):
        for j in range(n):
            common = 0
            while common < length and (t[i, common] == t[j, common]).all():
                common += 1
            for k in range(0, length, 9):
                assert (key(i, k) == key(j, k)) == (k < common)    # shared prefixes share their keys, and only those


def test_ladder_layout_makes_subtrees_contiguous():
    """All blocks below a prefix of 32 g blocks (512 g tokens) lie in the key range that the first 3 g bytes of the
    prefix's ladder span, and nothing else does: a range lookup under a long shared prefix is tight."""
    from workloads import keys as K
    toks = _prefix_tree_tokens(n_seq=80, length=100, seed=4)
    n, length = toks.shape[0], toks.shape[1]
    kb = _as_bytes(K.chain_keys(toks, "ladder"))
    t = toks.numpy()
    all_keys = sorted(set(kb))
    checked = 0
    for i in range(0, n, 3):
        for g in (1, 2, 3):
            deep = kb[i * length + 32 * g]                          # first block beyond the prefix of 32 g blocks
            lo, hi = deep[:3 * g] + bytes(32 - 3 * g), deep[:3 * g] + b"\xff" * (32 - 3 * g)
            inside = {k for k in all_keys if lo <= k <= hi}
            below = {kb[j * length + k] for j in range(n) if (t[j, :32 * g] == t[i, :32 * g]).all() for k in range(32 * g, length)}
            assert inside == below
            checked += 1
    assert checked > 50
    # the family layout does not have this property: a family's range also holds the blocks above the prefix
    fb = _as_bytes(K.chain_keys(toks, "family"))
    fam = fb[32][:8]
    assert any(k[:8] == fam and int.from_bytes(k[8:10], "big") < 32 for k in fb)
