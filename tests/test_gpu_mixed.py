"""Configuration 5 (mixed, shifting workload): the host driver with the GPU library as its
backend against the same driver with the CPU checker as its backend.  Every probe batch,
the sequence of compactions (sizes in and out), the policy decisions and the final tree
must be identical."""
import numpy as np
import pytest
import torch

from gpu_util import dev

pytestmark = pytest.mark.gpu


class OracleBackend:
    def __init__(self, oracle, stride=64):
        self.o, self.stride = oracle, stride

    def compact(self, runs, flags):
        return self.o.compact([self.o.as_run(r) for r in runs], flags & 1)

    def build_fences(self, run):
        return self.o.build_fences(self.o.as_run(run), self.stride)

    def probe(self, q, nb, tree):
        return self.o.probe(q, nb, [self.o.as_run(t.run) for t in tree])

    def hit_len_to_host(self, hit_len):
        return [int(x) for x in hit_len]

    def policy_choose(self, *a):
        return self.o.policy_choose(*a)


def _replay(backend, trace, runs, keep_probes, shuffle_writes=None):
    from paper_2511_16138_amd.tree import AdaptiveLsmTree, run_mixed_trace
    tree = AdaptiveLsmTree(backend, trace.buffer_entries, size_ratio=trace.size_ratio, window_ops=4 * trace.batch_requests)
    for level, r in enumerate(runs):
        tree.load_level(level, [r])
    run_mixed_trace(tree, trace, on_probe=lambda i, q, nb, out: keep_probes.append(out), shuffle_writes=shuffle_writes)
    return tree


@pytest.mark.parametrize("tree_total,buffer_entries,ops,shares,bloom_bits", [(400_000, 360, 4096, (0.9, 0.5, 0.1), 0),
                                                                             (2_000_000, 900, 8192, (0.9, 0.5, 0.02), 0),
                                                                             (400_000, 360, 4096, (0.9, 0.5, 0.1), 16),
                                                                             (400_000, 360, 4096, (0.9, 0.5, 0.1), -1)])
def test_mixed_trace_gpu_equals_checker(oracle, tree_total, buffer_entries, ops, shares, bloom_bits):
    from paper_2511_16138_amd.tree import GpuBackend
    from workloads import lsm
    print("mixed trace", tree_total, buffer_entries, ops, flush=True)
    tr = lsm.config5(device=dev(), tree_total=tree_total, buffer_entries=buffer_entries, ops_per_phase=ops, batch_requests=512, read_shares=shares)
    assert len([e for e in tr.events if e[0] == "flush"]) > 50 and len([e for e in tr.events if e[0] == "probe"]) >= 6

    gpu_probes, cpu_probes = [], []
    shuffle = None
    if bloom_bits < 0:  # the GPU side gets every write buffer in a random order and sorts it itself (lsm_flush_buffer)
        bloom_bits = 0
        shuffle = lambda i, n: torch.from_numpy(np.random.RandomState(i).permutation(n)).to(dev())
    gpu_tree = _replay(GpuBackend(bloom_bits=bloom_bits), tr, tr.workload.runs, gpu_probes, shuffle)  # the checker has no filters
    torch.cuda.synchronize()

    cpu_trace = lsm.MixedTrace(tr.workload, tr.buffer_entries, tr.size_ratio, tr.flush_runs.cpu(), tr.events, tr.batch_requests,
                               tr.write_ops_between)
    cpu_tree = _replay(OracleBackend(oracle), cpu_trace, [r.cpu() for r in tr.workload.runs], cpu_probes)

    assert gpu_tree.trace == cpu_tree.trace
    kinds = {e[0] for e in gpu_tree.trace}
    assert {"compact", "probe", "policy"} <= kinds
    ks = [e[2] for e in gpu_tree.trace if e[0] == "policy"]
    assert ks[0] == 1, ks  # leveling in the read-heavy phase
    if shares[2] < 0.05:   # with p = 1 and B = 64 the model leaves leveling only above ~93 % writes
        assert max(ks) > 1, ks
        assert any(e[0] == "compact" and e[2] > 2 for e in gpu_tree.trace)  # several runs per level were merged at once
    assert len(gpu_probes) == len(cpu_probes) > 0
    for (ghl, ghits), (chl, chits) in zip(gpu_probes, cpu_probes):
        assert np.array_equal(ghl.cpu().numpy().astype(np.uint32), chl)
        assert np.array_equal(ghits.cpu().numpy().view(oracle.HIT_DTYPE).reshape(chits.shape), chits)
    assert [len(lv) for lv in gpu_tree.levels] == [len(lv) for lv in cpu_tree.levels]
    for glv, clv in zip(gpu_tree.levels, cpu_tree.levels):
        for gr, cr in zip(glv, clv):
            assert np.array_equal(oracle.as_run(gr.run), oracle.as_run(cr.run))
            assert np.array_equal(gr.fences.cpu().numpy().view(np.uint8).reshape(-1, 32), cr.fences)
