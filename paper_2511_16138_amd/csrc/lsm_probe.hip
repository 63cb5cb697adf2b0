// lsm_probe: batched longest-cached-prefix lookup (paper appendix B, "Probe"; section 2.2,
// "Point Lookups": runs are checked newest to oldest and the first match is the result).
//
// One wave per request.  The request's block keys are handled 64 at a time, one key per
// lane: a lane walks the runs newest -> oldest, finds the page through the run's fence keys,
// searches the page, and stops at the first run that holds the key.  A ballot over the lanes
// gives the first block that is not live; later chunks of the request are then skipped.
#include <hip/hip_runtime.h>

#include "lsm_common.h"

namespace lsm {

struct TreeRun {
    const lsm_entry_t* entries;
    const uint8_t* fences;
    uint64_t n;
    uint64_t n_fences;
    uint32_t stride;
    uint32_t pad;
};

struct TreeTable {
    TreeRun run[LSM_MAX_RUNS];
    uint32_t n_runs;
};

constexpr int kProbeThreads = 256;

// Index of the entry with this key in the run, or ~0 if absent.
__device__ __forceinline__ uint64_t find_in_run(const TreeRun& tr, const Key& q) {
    // page = last fence <= q
    uint64_t lo = 0, hi = tr.n_fences;
    while (lo < hi) {
        uint64_t mid = lo + ((hi - lo) >> 1);
        if (key_less(q, load_key(tr.fences + mid * LSM_KEY_BYTES))) hi = mid;
        else lo = mid + 1;
    }
    if (lo == 0) return ~0ull;  // q is below the first key of the run
    uint64_t first = (lo - 1) * (uint64_t)tr.stride;
    uint64_t last = first + tr.stride < tr.n ? first + tr.stride : tr.n;
    uint64_t i = lower_bound_run(tr.entries, first, last, q);
    if (i < last && key_equal(load_key(tr.entries + i), q)) return i;
    return ~0ull;
}

__global__ void __launch_bounds__(kProbeThreads) probe_kernel(TreeTable tree, const uint8_t* qkeys, const uint32_t* n_blocks,
                                                               uint32_t n_req, uint32_t max_blocks, uint32_t* hit_len,
                                                               lsm_hit_t* hits) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint32_t req = blockIdx.x * (kProbeThreads / kWave) + threadIdx.x / kWave;
    if (req >= n_req) return;  // whole wave
    uint32_t nb = n_blocks[req];
    if (nb > max_blocks) nb = max_blocks;
    const uint8_t* qrow = qkeys + (uint64_t)req * max_blocks * LSM_KEY_BYTES;
    uint4* hrow = reinterpret_cast<uint4*>(hits + (uint64_t)req * max_blocks);
    uint32_t result = nb;
    bool done = false;
    for (uint32_t c0 = 0; c0 < max_blocks; c0 += kWave) {
        const uint32_t j = c0 + lane;
        uint4 h = make_uint4(0, 0, 0, 0);
        if (!done && c0 < nb) {
            bool live = true;  // lanes past the request's length do not end the prefix
            if (j < nb) {
                live = false;
                Key q = load_key(qrow + (uint64_t)j * LSM_KEY_BYTES);
                for (uint32_t r = 0; r < tree.n_runs; r++) {
                    uint64_t i = find_in_run(tree.run[r], q);
                    if (i != ~0ull) {
                        const uint4* e = reinterpret_cast<const uint4*>(tree.run[r].entries + i);
                        uint4 meta = e[2], val = e[3];  // seqno | type+pad, vptr | vlen+pad
                        if ((meta.z & 0xFF) == LSM_PUT) {
                            live = true;
                            h = make_uint4(val.x, val.y, val.z, r);
                        }
                        break;
                    }
                }
            }
            uint64_t dead = __ballot(!live);
            if (dead) {
                uint32_t first = (uint32_t)__ffsll((unsigned long long)dead) - 1;
                result = c0 + first;
                done = true;
                if ((uint32_t)lane >= first) h = make_uint4(0, 0, 0, 0);
            }
        }
        if (j < max_blocks) hrow[j] = h;
    }
    if (lane == 0) hit_len[req] = result;
}

}  // namespace lsm

extern "C" int lsm_probe(const lsm_queries_t* queries, const lsm_tree_t* tree, const lsm_hits_t* out_hits, void* stream) {
    using namespace lsm;
    if (queries == nullptr || tree == nullptr || out_hits == nullptr) return LSM_ERR_NULL;
    if (queries->max_blocks == 0 || queries->max_blocks > LSM_MAX_BLOCKS || tree->n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    if (queries->n_req == 0) return LSM_OK;
    if (queries->keys == nullptr || queries->n_blocks == nullptr || out_hits->hit_len == nullptr || out_hits->hits == nullptr)
        return LSM_ERR_NULL;
    if (tree->n_runs > 0 && tree->runs == nullptr) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(queries->keys) & 15) != 0 || (reinterpret_cast<uintptr_t>(out_hits->hits) & 15) != 0)
        return LSM_ERR_BAD_ARG;
    TreeTable tt;
    tt.n_runs = 0;
    for (uint32_t r = 0; r < tree->n_runs; r++) {
        const lsm_tree_run_t& tr = tree->runs[r];
        TreeRun& d = tt.run[r];
        d.entries = tr.run.entries;
        d.n = tr.run.n;
        d.fences = tr.fence.keys;
        d.n_fences = tr.fence.n;
        d.stride = tr.fence.stride;
        d.pad = 0;
        if (tr.run.n > 0) {
            if (tr.run.entries == nullptr || tr.fence.keys == nullptr) return LSM_ERR_NULL;
            if (tr.fence.stride == 0 || tr.fence.n != (tr.run.n + tr.fence.stride - 1) / tr.fence.stride) return LSM_ERR_BAD_ARG;
            if ((reinterpret_cast<uintptr_t>(tr.run.entries) & 63) != 0 || (reinterpret_cast<uintptr_t>(tr.fence.keys) & 15) != 0)
                return LSM_ERR_BAD_ARG;
        } else {
            d.n_fences = 0;  // an empty run is never searched
        }
    }
    tt.n_runs = tree->n_runs;
    for (uint32_t r = tree->n_runs; r < LSM_MAX_RUNS; r++) tt.run[r] = TreeRun{nullptr, nullptr, 0, 0, 1, 0};
    const uint32_t per_block = kProbeThreads / kWave;
    uint32_t blocks = (queries->n_req + per_block - 1) / per_block;
    hipLaunchKernelGGL(probe_kernel, dim3(blocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), tt, queries->keys,
                       queries->n_blocks, queries->n_req, queries->max_blocks, out_hits->hit_len, out_hits->hits);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
