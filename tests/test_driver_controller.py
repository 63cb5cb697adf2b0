"""The controller of the library's driver (lsm_driver_note_writes / lsm_driver_note_reads: sliding window, threshold,
(T, K) search, log) on the CPU: no run is loaded, so nothing touches a GPU.  Checked against a scenario worked out by
hand and, on random operation streams, against the plain driver of oracle/lsm_driver_oracle.py."""
import math

import numpy as np
import pytest


@pytest.fixture(scope="module")
def LsmDriver():
    import os
    import paper_2511_16138_amd.binding as B
    if not os.path.exists(B.library_path()):
        import __graft_entry__
        __graft_entry__.build()
    return B.LsmDriver


def test_window_slides_and_threshold_holds(LsmDriver):
    d = LsmDriver(100, size_ratio=10, window_ops=100, shift_threshold=0.2, t_grid=(10, 10), filter_fpr=1.0)
    for _ in range(9):
        d.note_writes(10)
    assert d.trace == []                        # 90 operations: the window is not full
    d.note_writes(10)
    assert len(d.trace) == 1 and d.trace[0][0] == "policy" and d.trace[0][3] == (1.0, 0.0, 0.0, 0.0)
    d.note_reads(5, 4, 50)                      # 9 % reads: moved by 0.18 in L1 distance -> below the threshold
    assert [e[0] for e in d.trace] == ["policy", "probe"] and d.trace[1] == ("probe", 9, 5, 50)
    d.note_reads(2, 1, 20)                      # 3 + 9 + 9 x 10 = 102 >= 100: the oldest write batch leaves the window
    # mix (90, 7/2, 7/2, 5) / 102: moved by 12/102 + 7/102 + 5/102 = 0.235 -> a second search, d = 70 blocks / 7 requests
    assert [e[0] for e in d.trace] == ["policy", "probe", "probe", "policy"]
    _, T, K, mix, dd = d.trace[3]
    assert T == 10 and 1 <= K <= 9
    assert mix == (round(90 / 102, 6), round(3.5 / 102, 6), round(3.5 / 102, 6), round(5 / 102, 6)) and dd == 10.0
    assert d.target() == (T, K) and d.levels() == []
    d.close()


def test_all_writes_choose_tiering_all_reads_choose_leveling(LsmDriver):
    # N = 1 entry, so one level: W = T / (B K) is smallest for K = T - 1 at the largest T (8 / 7 < 7 / 6 < ...);
    # the lookup costs K + d / B and K p + 1 grow with K and do not depend on T, and ties go to the smaller T
    d = LsmDriver(100, window_ops=10, t_grid=(2, 8), filter_fpr=1.0)
    d.note_writes(10)
    assert d.trace[-1][:3] == ("policy", 8, 7)
    d.note_reads(10, 0, 10)                    # the writes leave the window at once: 10 reads cover it
    assert d.trace[-1][:3] == ("policy", 2, 1) and d.trace[-1][3] == (0.0, 0.5, 0.5, 0.0) and d.trace[-1][4] == 1.0
    d.note_reads(10, 0, 10)                    # the same mix again: no new search
    assert [e[0] for e in d.trace] == ["policy", "probe", "policy", "probe"]
    d.close()


@pytest.mark.parametrize("seed,window,threshold,t_grid,bits", [
    (1, 1000, 0.2, (2, 16), 16), (2, 64, 0.05, (2, 16), 0), (3, 5000, 0.5, (10, 10), 16), (4, 1, 0.0, (3, 7), 8), (5, 300, 0.2, (2, 4), 16)])
def test_controller_follows_the_plain_driver_on_random_streams(LsmDriver, seed, window, threshold, t_grid, bits):
    from oracle import lsm_driver_oracle as drv
    rs = np.random.RandomState(seed)
    d = LsmDriver(3600, size_ratio=10, window_ops=window, shift_threshold=threshold, t_grid=t_grid, bloom_bits=bits)
    c = drv.DriverOracle(3600, T=10, K=1, window_ops=window, threshold=threshold, t_grid=t_grid, page_entries=64.0, fpr=drv.bloom_fpr(bits))
    for phase in range(6):
        read_share = rs.rand()                   # the mix shifts from phase to phase
        for _ in range(100):
            if rs.rand() >= read_share:
                n = int(rs.randint(0, 400))
                d.note_writes(n)
                c.writes(n)
            else:
                ok, empty = int(rs.randint(0, 200)), int(rs.randint(0, 200))
                blocks = ok * int(rs.randint(1, 40))
                d.note_reads(ok, empty, blocks)
                c.observe_reads(ok, empty, blocks)
            assert len(d.trace) == len(c.log)
    assert d.trace == c.log and d.target() == (c.target_T, c.target_K)
    assert sum(1 for e in c.log if e[0] == "policy") >= 2
    if t_grid == (2, 16):
        assert len({e[1:3] for e in c.log if e[0] == "policy"}) > 1     # the choice moves with the mix
    assert math.isclose(c.p, drv.bloom_fpr(bits))
    d.close()
