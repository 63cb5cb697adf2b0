"""lsm_compact_static (the entry point that allocates nothing) against lsm_compact: same bytes, same count, on two
calls in a row that share the library's static scratch, the second with a smaller input."""
import numpy as np
import pytest
import torch

from gpu_util import as_bytes, dev

pytestmark = pytest.mark.gpu


def _both(g, runs, flags):
    total = sum(int(r.shape[0]) for r in runs)
    want, want_n = g.lsm_compact(runs, flags)
    out = torch.full((max(total, 1), 8), -1, dtype=torch.int64, device=dev())
    n_out = torch.full((1,), -7, dtype=torch.int64, device=dev())
    fences = torch.zeros(((total + 63) // 64 + 1, 4), dtype=torch.int64, device=dev())
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    g.lsm_compact_static(runs, flags, out, n_out, fences=fences, fence_stride=64)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    n = int(n_out.item())
    assert n == int(want_n.item())
    assert np.array_equal(as_bytes(out[:n]), as_bytes(want[:n]))
    if n:
        assert np.array_equal(as_bytes(fences[: (n + 63) // 64]), as_bytes(g.lsm_build_fences(want[:n].contiguous(), 64)))
    return n


def test_static_scratch_compaction_equals_lsm_compact(oracle):
    import paper_2511_16138_amd as g
    from workloads import lsm
    big = lsm.config3(device=dev(), scale=16)     # 16 runs x 262,144 entries: 2,065 tiles, the sampled partition
    print("static scratch: first call", sum(int(r.shape[0]) for r in big.runs), flush=True)
    n_big = _both(g, [r.contiguous() for r in big.runs], g.LSM_BOTTOMMOST)
    small = lsm.config1(device=dev())             # 4 runs, 65,536 entries: the direct partition, far fewer tiles
    print("static scratch: second call", sum(int(r.shape[0]) for r in small.runs), flush=True)
    runs = [r.contiguous() for r in small.runs]
    n_small = _both(g, runs, 0)
    assert 0 < n_small < n_big
    want = oracle.compact([r.cpu() for r in small.runs], 0)   # and the small one against the CPU checker as well
    out = torch.empty((65536, 8), dtype=torch.int64, device=dev())
    n_out = torch.zeros(1, dtype=torch.int64, device=dev())
    g.lsm_compact_static(runs, 0, out, n_out)
    assert np.array_equal(oracle.as_run(out[: int(n_out.item())]), want)
    _both(g, [runs[0][:0], runs[1][:5]], g.LSM_BOTTOMMOST)    # third call: almost nothing


def test_static_scratch_limit_is_an_error():
    import paper_2511_16138_amd as g
    n = 1 << 24   # 16M entries need about 16 MB of scratch: beyond the 8 MiB array
    run = torch.zeros((n, 8), dtype=torch.int64, device=dev())
    out = torch.empty((n, 8), dtype=torch.int64, device=dev())
    n_out = torch.full((1,), 5, dtype=torch.int64, device=dev())
    with pytest.raises(g.LsmError) as e:
        g.lsm_compact_static([run], 0, out, n_out)
    assert e.value.code == -9 and int(n_out.item()) == 5
