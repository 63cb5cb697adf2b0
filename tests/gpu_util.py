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


def oracle_probe_threads(oracle, q, nb, runs, threads=16):
    """oracle.probe with the requests split over threads (the C checker runs without the interpreter lock).  The
    arithmetic is the checker's; only the batch is cut into slices and the results are put back together."""
    from concurrent.futures import ThreadPoolExecutor
    if hasattr(q, "detach"):
        q = q.detach().cpu().contiguous().numpy()
    if hasattr(nb, "detach"):
        nb = nb.detach().cpu().numpy()
    n = int(nb.shape[0])
    q = np.ascontiguousarray(q).view(np.uint8).reshape(n, -1, 32)
    runs = [oracle.as_run(r) for r in runs]
    cuts = np.linspace(0, n, min(threads, max(n, 1)) + 1).astype(np.int64)
    parts = [(int(a), int(b)) for a, b in zip(cuts[:-1], cuts[1:]) if b > a]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        res = list(ex.map(lambda ab: oracle.probe(q[ab[0]:ab[1]], nb[ab[0]:ab[1]], runs), parts))
    if not res:
        return oracle.probe(q, nb, runs)
    return np.concatenate([r[0] for r in res]), np.concatenate([r[1] for r in res])
