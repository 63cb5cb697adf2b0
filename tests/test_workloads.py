"""Properties of the seeded input generator (CPU only)."""
import numpy as np
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
