"""Helpers shared by the GPU parity tests (all calls go through the C ABI binding)."""
import numpy as np
import torch


def dev():
    return torch.device("cuda:0")


def to_dev(run_np):
    """uint8 [n, 64] numpy -> int64 [n, 8] GPU tensor."""
    a = np.ascontiguousarray(run_np).view(np.int64).reshape(-1, 8)
    return torch.from_numpy(a.copy()).to(dev())


def compact_gpu(g, runs, flags):
    out, n_out = g.lsm_compact(runs, flags)
    torch.cuda.synchronize()
    n = int(n_out.item())
    assert 0 <= n <= out.shape[0], f"n_out = {n}"
    return out[:n]


def as_bytes(t):
    return t.detach().cpu().contiguous().numpy().view(np.uint8)


def build_tree(g, runs, stride=64):
    return [g.TreeRun(r.contiguous(), g.lsm_build_fences(r.contiguous(), stride), stride, i) for i, r in enumerate(runs)]


def probe_gpu(g, q, nb, tree):
    hit_len, hits = g.lsm_probe(q, nb, tree)
    torch.cuda.synchronize()
    return hit_len.cpu().numpy().astype(np.uint32), hits.cpu().numpy()


def assert_probe_equal(oracle, got, want):
    hl, hits = got
    whl, whits = want
    assert np.array_equal(hl, whl)
    assert np.array_equal(hits.view(oracle.HIT_DTYPE).reshape(whits.shape), whits)
