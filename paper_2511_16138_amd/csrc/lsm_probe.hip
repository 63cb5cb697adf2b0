// lsm_probe: batched longest-cached-prefix lookup (paper appendix B, "Probe"; section 2.2,
// "Point Lookups": runs are checked newest to oldest and the first match is the result).
//
// One wave per request, requests taken round-robin by the waves of a fixed-size grid.  Every
// workgroup first copies a top-level fence table into LDS: for each run of the tree, an evenly
// spaced subset of its fence keys (all of them for small runs).  A request's block keys are
// handled 64 at a time, one key per lane.  A lane first reads the Bloom filters of the runs that have one
// (all together), then walks the runs they admit, newest -> oldest, each lane its own list, and stops at
// the first run that holds the key: top-level fences in LDS, then the remaining fence range and the
// 64-entry page in global memory, reading the first 16 key bytes and the second half only on a tie.
// A ballot over the lanes gives the first block that is not live; later chunks of the request are
// skipped and zero-filled.
#include <hip/hip_runtime.h>

#include "lsm_common.h"

namespace lsm {

struct TreeRun {
    const lsm_entry_t* entries;
    const uint8_t* fences;  // ceil(n / stride) keys
    uint64_t n;
    const uint64_t* index;  // hash index of index_buckets(n) buckets, or null
    uint32_t stride;
    uint32_t bloom_blocks;  // 0 = no filter
    const uint4* bloom;
};
static_assert(sizeof(TreeRun) == 48, "64 of these travel as a kernel argument");

struct TreeTable {
    TreeRun run[LSM_MAX_RUNS];
    uint32_t n_runs;
};

constexpr int kProbeThreads = 256;
constexpr int kProbeWays = 3;     // fan-out of a search step in global memory (measured: 2: 0.072 ms per batch, 3: 0.067, 4: 0.069, 6: 0.074, 8: 0.080)
constexpr int kTopSlots = 1024;  // top-level fence keys held in LDS per workgroup (32 KB)

struct ProbeShared {
    uint4 top_lo[kTopSlots];  // first 16 bytes of each top-level fence key
    uint4 top_hi[kTopSlots];  // last 16 bytes
    uint32_t first_slot[LSM_MAX_RUNS];  // slots of run r: [first_slot[r], first_slot[r] + n_top[r])
    uint32_t n_top[LSM_MAX_RUNS];
    uint32_t top_stride[LSM_MAX_RUNS];  // top key i of run r = fence i * top_stride[r]
    // the run descriptors, readable with a per-lane run number
    const uint8_t* fences[LSM_MAX_RUNS];
    const lsm_entry_t* entries[LSM_MAX_RUNS];
    uint64_t n[LSM_MAX_RUNS];
    uint64_t n_fences[LSM_MAX_RUNS];
    uint32_t stride[LSM_MAX_RUNS];
    const uint64_t* index[LSM_MAX_RUNS];  // hash index of the run, or null
};

// -1 / 0 / +1 for q < / == / > the 32-byte key whose halves are (lo, hi); hi is only fetched on a tie
template <typename LoadHi>
__device__ __forceinline__ int compare_key(const Key& q, uint4 lo, LoadHi load_hi) {
    const uint64_t w0 = __builtin_bswap64(((uint64_t)lo.y << 32) | lo.x);
    const uint64_t w1 = __builtin_bswap64(((uint64_t)lo.w << 32) | lo.z);
    if (q.w[0] != w0) return q.w[0] < w0 ? -1 : 1;
    if (q.w[1] != w1) return q.w[1] < w1 ? -1 : 1;
    const uint4 hi = load_hi();
    const uint64_t w2 = __builtin_bswap64(((uint64_t)hi.y << 32) | hi.x);
    const uint64_t w3 = __builtin_bswap64(((uint64_t)hi.w << 32) | hi.z);
    if (q.w[2] != w2) return q.w[2] < w2 ? -1 : 1;
    if (q.w[3] != w3) return q.w[3] < w3 ? -1 : 1;
    return 0;
}

// Copies the run descriptors and, with kTop, the top-level fence table into LDS (all threads of the workgroup call this).
// Without the table (every run has a hash index, so the fences are only searched for keys of crowded buckets) a fence
// search starts from the whole fence array.
template <bool kTop>
__device__ __forceinline__ void probe_setup(ProbeShared& s, const TreeTable& tree, const int tid) {
    const uint32_t n_runs = tree.n_runs;
    // ---- top-level fence table: an equal share of the slots for every run
    const uint32_t share = (kTop && n_runs) ? kTopSlots / n_runs : 0;
    if (tid < (int)n_runs) {
        const uint32_t stride = tree.run[tid].stride;  // >= 1 (checked by the host)
        const uint64_t nf = (tree.run[tid].n + stride - 1) / stride;
        const uint32_t ts = share ? (uint32_t)((nf + share - 1) / share) : 1;
        s.first_slot[tid] = tid * share;
        s.top_stride[tid] = ts ? ts : 1;
        s.n_top[tid] = ts ? (uint32_t)((nf + ts - 1) / ts) : 0;
        s.fences[tid] = tree.run[tid].fences;
        s.entries[tid] = tree.run[tid].entries;
        s.n[tid] = tree.run[tid].n;
        s.n_fences[tid] = nf;
        s.stride[tid] = stride;
        s.index[tid] = tree.run[tid].index;
    }
    __syncthreads();
    if (kTop) {
        for (uint32_t slot = tid; slot < share * n_runs; slot += kProbeThreads) {
            const uint32_t r = slot / share, i = slot - r * share;
            if (i < s.n_top[r]) {
                const uint4* f = reinterpret_cast<const uint4*>(tree.run[r].fences + (uint64_t)i * s.top_stride[r] * LSM_KEY_BYTES);
                s.top_lo[slot] = f[0];
                s.top_hi[slot] = f[1];
            }
        }
        __syncthreads();
    }
}

// Whether a key with this tag can be in the bucket whose tag fields are w: some field carries the tag, or the bucket is crowded
__device__ __forceinline__ bool index_admits(const uint4 w, const uint32_t tag) {
    const uint32_t x[4] = {w.x, w.y, w.z, w.w};
    bool any = (w.x & 0x8000u) != 0;
#pragma unroll
    for (int i = 0; i < 4; i++) any = any || (x[i] & kIndexTagMask) == tag || ((x[i] >> 16) & kIndexTagMask) == tag;
    return any;
}

// Looks one block key per lane up in the tree (every lane of the wave calls this; lanes with mine == false idle).
// Returns whether the key's newest version is a live PUT (true for idle lanes) and sets h to its hit record.
template <bool kTop>
__device__ __forceinline__ bool probe_lookup(const ProbeShared& s, const TreeTable& tree, const uint32_t n_runs,
                                             const uint64_t run_mask, const bool any_filter, const bool mine, const Key& q, uint4& h) {
    bool live = !mine, found = !mine;
    // (0) Bloom filters of the runs that have one: one 16-byte read per run, all runs of a group of
    //     eight requested together, decides which runs this key is searched in
    uint64_t maybe = ~0ull;
    const uint64_t bh = mine ? bloom_key_hash(q) : 0;
    const uint32_t tag = (uint32_t)bh & kIndexTagMask;
    if (mine && any_filter) {
        // one 16-byte read per run: the tags of the key's bucket in the run's hash index, else the key's filter block
        const uint4 mask = bloom_mask(bh);
        for (uint32_t rb = 0; rb < n_runs; rb += 8) {
            uint4 w[8];
#pragma unroll
            for (int g = 0; g < 8; g++) {
                const uint32_t r = rb + g;
                w[g] = make_uint4(~0u, ~0u, ~0u, ~0u);
                if (r < n_runs) {
                    // a run that has both is asked through its filter: an eighth of the index's size, so far more of it
                    // stays in the caches
                    if (tree.run[r].bloom_blocks != 0)
                        w[g] = tree.run[r].bloom[bloom_block(bh, tree.run[r].bloom_blocks)];
                    else if (tree.run[r].index != nullptr)
                        w[g] = reinterpret_cast<const uint4*>(tree.run[r].index)[(uint64_t)bloom_block(bh, (uint32_t)index_buckets(tree.run[r].n)) * 4];
                }
            }
#pragma unroll
            for (int g = 0; g < 8; g++) {
                const uint32_t r = rb + g;
                bool out;
                if (r < n_runs && tree.run[r].bloom_blocks == 0 && tree.run[r].index != nullptr) out = !index_admits(w[g], tag);
                else out = bloom_excludes(w[g], mask);
                if (out) maybe &= ~(1ull << r);
            }
        }
    }
    maybe &= run_mask;
    // every lane walks its own list of admitted runs, newest first, so lanes that need different
    // runs search them at the same time; the walk of a lane ends at the first run that holds its key
    while (__ballot(!found && maybe != 0) != 0) {
        const bool act = !found && maybe != 0;
        const uint32_t r = act ? (uint32_t)__builtin_ctzll(maybe) : 0;
        maybe &= maybe - 1;  // 0 stays 0
        // (0b) a run with a hash index: the key's bucket holds its tag and position (the line was read in step 0, so
        //      this read stays in the caches); only a key of a crowded bucket that is not among the bucket's eight goes
        //      on to the fences
        bool via_fences = act;
        const uint64_t* index = act ? s.index[r] : nullptr;
        if (index != nullptr) {
            const uint64_t n = s.n[r];
            const uint4* bucket = reinterpret_cast<const uint4*>(index) + (uint64_t)bloom_block(bh, (uint32_t)index_buckets(n)) * 4;
            const uint4 t = bucket[0], p0 = bucket[1], p1 = bucket[2];
            const uint32_t pos[kIndexSlots] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
            const uint32_t field[kIndexSlots] = {t.x & 0xFFFF, t.x >> 16, t.y & 0xFFFF, t.y >> 16, t.z & 0xFFFF, t.z >> 16, t.w & 0xFFFF, t.w >> 16};
            via_fences = (t.x & 0x8000u) != 0;  // crowded
            uint32_t same = 0;
#pragma unroll
            for (int k = 0; k < (int)kIndexSlots; k++) same |= (pos[k] != kIndexNoEntry && (field[k] & kIndexTagMask) == tag) ? 1u << k : 0u;
            while (same != 0) {  // nearly always one candidate at most: another needs a second key with the same tag
                const int k = __builtin_ctz(same);
                same &= same - 1;
                uint32_t at = pos[0];
#pragma unroll
                for (int j = 1; j < (int)kIndexSlots; j++) at = k == j ? pos[j] : at;
                if (at >= n) continue;  // a table that does not belong to the run must not send a read outside it
                const uint4* e = reinterpret_cast<const uint4*>(s.entries[r] + at);
                const uint4 k0 = e[0], k1 = e[1], meta = e[2], val = e[3];
                if (compare_key(q, k0, [&] { return k1; }) == 0) {
                    found = true;
                    via_fences = false;
                    same = 0;
                    if ((meta.z & 0xFF) == LSM_PUT) {
                        live = true;
                        h = make_uint4(val.x, val.y, val.z, r);
                    }
                }
            }
        }
        // (1) top-level fences in LDS: number of top keys <= q
        uint32_t lo = 0, hi = (kTop && via_fences) ? s.n_top[r] : 0;
        const uint32_t first_slot = s.first_slot[r];
        while (__ballot(lo < hi) != 0) {
            if (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1, slot = first_slot + mid;
                const int c = compare_key(q, s.top_lo[slot], [&] { return s.top_hi[slot]; });
                if (c < 0) hi = mid;
                else lo = mid + 1;
            }
        }
        // (2) the fences between two top keys, in global memory: number of fences <= q
        const uint8_t* fences = s.fences[r];
        if (!kTop) {  // no table: the whole fence array
            lo = 0;
            hi = via_fences ? (uint32_t)s.n_fences[r] : 0;
        } else if (lo > 0) {  // lo = top keys <= q; 0 means q is below the run's first key (or the lane is idle)
            const uint32_t ts = s.top_stride[r];
            const uint64_t nf = s.n_fences[r], end = (uint64_t)lo * ts;
            hi = (uint32_t)(end < nf ? end : nf);
            lo = (lo - 1) * ts + 1;  // fence (lo-1)*ts is <= q
        } else {
            hi = 0;
        }
        // kProbeWays-way steps: kProbeWays - 1 fence keys are requested together, fewer dependent round trips than
        // bisection for more reads; the kernel is bound by both, and the fan-out is the measured optimum
        while (__ballot(lo < hi) != 0) {
            if (lo < hi) {
                const uint32_t w = hi - lo;
                uint4 a[kProbeWays - 1];
                uint32_t m[kProbeWays - 1];
#pragma unroll
                for (int i = 0; i < kProbeWays - 1; i++) {
                    m[i] = lo + (uint32_t)(((uint64_t)(i + 1) * w) / kProbeWays);  // lo <= m[0] <= ... <= m[last] < hi
                    a[i] = *reinterpret_cast<const uint4*>(fences + (uint64_t)m[i] * LSM_KEY_BYTES);
                }
                // number of fences <= q: the last probed fence that is <= q bounds it from below, the first one that
                // is > q from above (the answers are monotone along the probes)
                uint32_t new_lo = lo, new_hi = hi;
#pragma unroll
                for (int i = kProbeWays - 2; i >= 0; i--) {
                    const uint8_t* f = fences + (uint64_t)m[i] * LSM_KEY_BYTES;
                    const int c = compare_key(q, a[i], [&] { return *reinterpret_cast<const uint4*>(f + 16); });
                    if (c >= 0) new_lo = max(new_lo, m[i] + 1);
                    else new_hi = m[i];
                }
                lo = new_lo;
                hi = new_hi;
            }
        }
        // (3) the page of the last fence <= q: first entry whose key is >= q
        const lsm_entry_t* page = s.entries[r];
        uint32_t page_len = 0;
        if (lo > 0) {  // lo = fences <= q
            const uint32_t stride = s.stride[r];
            const uint64_t start = (uint64_t)(lo - 1) * stride, left = s.n[r] - start;
            page += start;
            page_len = (uint32_t)(left < stride ? left : stride);
        }
        lo = 0;
        hi = page_len;
        while (__ballot(lo < hi) != 0) {
            if (lo < hi) {
                const uint32_t w = hi - lo;
                uint4 a[kProbeWays - 1];
                uint32_t m[kProbeWays - 1];
#pragma unroll
                for (int i = 0; i < kProbeWays - 1; i++) {
                    m[i] = lo + (uint32_t)(((uint64_t)(i + 1) * w) / kProbeWays);
                    a[i] = reinterpret_cast<const uint4*>(page + m[i])[0];
                }
                // first entry whose key is >= q
                uint32_t new_lo = lo, new_hi = hi;
#pragma unroll
                for (int i = kProbeWays - 2; i >= 0; i--) {
                    const uint4* e = reinterpret_cast<const uint4*>(page + m[i]);
                    const int c = compare_key(q, a[i], [&] { return e[1]; });
                    if (c > 0) new_lo = max(new_lo, m[i] + 1);
                    else new_hi = m[i];
                }
                lo = new_lo;
                hi = new_hi;
            }
        }
        // (4) is it there?  The four parts of the candidate are requested together (one 64-byte line).
        if (lo < page_len) {
            const uint4* e = reinterpret_cast<const uint4*>(page + lo);
            const uint4 k0 = e[0], k1 = e[1], meta = e[2], val = e[3];  // key | seqno, type + pad | vptr, vlen + pad
            if (compare_key(q, k0, [&] { return k1; }) == 0) {
                found = true;
                if ((meta.z & 0xFF) == LSM_PUT) {
                    live = true;
                    h = make_uint4(val.x, val.y, val.z, r);
                }
            }
        }
    }
    return live;
}

template <bool kTop>
__global__ void __launch_bounds__(kProbeThreads) probe_kernel(TreeTable tree, const uint8_t* qkeys, const uint32_t* n_blocks,
                                                               uint32_t n_req, uint32_t max_blocks, uint32_t* hit_len,
                                                               lsm_hit_t* hits) {
    __shared__ ProbeShared s;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const uint32_t n_runs = tree.n_runs;
    probe_setup<kTop>(s, tree, tid);
    const uint64_t run_mask = n_runs >= 64 ? ~0ull : (1ull << n_runs) - 1;
    bool any_filter = false;  // a Bloom filter or a hash index
    for (uint32_t r = 0; r < n_runs; r++) any_filter = any_filter || tree.run[r].bloom_blocks != 0 || tree.run[r].index != nullptr;
    const uint32_t waves = gridDim.x * (kProbeThreads / kWave);
    for (uint32_t req = blockIdx.x * (kProbeThreads / kWave) + tid / kWave; req < n_req; req += waves) {
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
                const bool mine = j < nb;  // lanes past the request's length do not end the prefix
                Key q = {{0, 0, 0, 0}};
                if (mine) q = load_key(qrow + (uint64_t)j * LSM_KEY_BYTES);
                const bool live = probe_lookup<kTop>(s, tree, n_runs, run_mask, any_filter, mine, q, h);
                const uint64_t dead = __ballot(!live);
                if (dead) {
                    const uint32_t first = (uint32_t)__ffsll((unsigned long long)dead) - 1;
                    result = c0 + first;
                    done = true;
                    if ((uint32_t)lane >= first) h = make_uint4(0, 0, 0, 0);
                }
            }
            if (j < max_blocks) hrow[j] = h;
        }
        if (lane == 0) hit_len[req] = result;
    }
}

// The length of the longest cached prefix by a search over the prefix length (appendix B, "Probe") instead of a
// lookup of every block key: valid when the tree is prefix-closed (block j of a request live => blocks 0..j-1
// live).  One wave per request, two rounds: 64 evenly spaced blocks, then the blocks between the last live and the
// first dead one of those.
template <bool kTop>
__global__ void __launch_bounds__(kProbeThreads) probe_length_kernel(TreeTable tree, const uint8_t* qkeys, const uint32_t* n_blocks,
                                                                      uint32_t n_req, uint32_t max_blocks, uint32_t* hit_len) {
    __shared__ ProbeShared s;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const uint32_t n_runs = tree.n_runs;
    probe_setup<kTop>(s, tree, tid);
    const uint64_t run_mask = n_runs >= 64 ? ~0ull : (1ull << n_runs) - 1;
    bool any_filter = false;  // a Bloom filter or a hash index
    for (uint32_t r = 0; r < n_runs; r++) any_filter = any_filter || tree.run[r].bloom_blocks != 0 || tree.run[r].index != nullptr;
    const uint32_t waves = gridDim.x * (kProbeThreads / kWave);
    for (uint32_t req = blockIdx.x * (kProbeThreads / kWave) + tid / kWave; req < n_req; req += waves) {
        uint32_t nb = n_blocks[req];
        if (nb > max_blocks) nb = max_blocks;
        const uint8_t* qrow = qkeys + (uint64_t)req * max_blocks * LSM_KEY_BYTES;
        uint32_t lo = 0, hi = nb;  // blocks below lo are live, block hi is not (or hi == nb)
        while (lo < hi) {
            // lane l asks for block lo + (l + 1) * step - 1, the last lane that has one for block hi - 1
            const uint32_t span = hi - lo, step = (span + kWave - 1) / kWave, lanes = (span + step - 1) / step;
            const bool mine = (uint32_t)lane < lanes;
            uint32_t j = lo + ((uint32_t)lane + 1) * step - 1;
            if (j > hi - 1) j = hi - 1;
            Key q = {{0, 0, 0, 0}};
            if (mine) q = load_key(qrow + (uint64_t)j * LSM_KEY_BYTES);
            uint4 h;
            const bool live = probe_lookup<kTop>(s, tree, n_runs, run_mask, any_filter, mine, q, h);
            const uint64_t dead = __ballot(!live);
            if (dead == 0) {
                lo = hi;  // block hi - 1 is live: so is everything below it
            } else {
                const uint32_t first = (uint32_t)__ffsll((unsigned long long)dead) - 1;  // first lane whose block is not live
                uint32_t dead_at = lo + (first + 1) * step - 1;
                if (dead_at > hi - 1) dead_at = hi - 1;
                hi = dead_at;
                lo = lo + first * step;  // the block of lane first - 1 (or everything below lo) is live
            }
        }
        if (lane == 0) hit_len[req] = lo;
    }
}

// One thread per (run, bound): entries of the run below the key, by bisection over the run itself.
__global__ void range_bounds_kernel(TreeTable tree, Key lo_key, Key hi_key, uint64_t* bounds) {
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= 2 * tree.n_runs) return;
    const TreeRun& run = tree.run[t >> 1];
    bool eq;
    bounds[t] = run.n ? lower_bound_eq(run.entries, 0, run.n, (t & 1) ? hi_key : lo_key, eq) : 0;
}

}  // namespace lsm

// Checks a tree descriptor and copies it into the by-value table the kernels take.
// Whether the kernels can do without the top-level fence table: every run that holds entries has a hash index.
static bool all_indexed(const lsm::TreeTable& tt) {
    bool any = false;
    for (uint32_t r = 0; r < tt.n_runs; r++) {
        if (tt.run[r].n == 0) continue;
        if (tt.run[r].index == nullptr) return false;
        any = true;
    }
    return any;
}

static int make_tree_table(const lsm_tree_t* tree, lsm::TreeTable& tt) {
    using namespace lsm;
    if (tree->n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    if (tree->n_runs > 0 && tree->runs == nullptr) return LSM_ERR_NULL;
    tt.n_runs = 0;
    for (uint32_t r = 0; r < tree->n_runs; r++) {
        const lsm_tree_run_t& tr = tree->runs[r];
        TreeRun& d = tt.run[r];
        d.entries = tr.run.entries;
        d.n = tr.run.n;
        d.fences = tr.fence.keys;
        d.stride = tr.fence.stride;
        d.index = static_cast<const uint64_t*>(tr.index.buckets);
        if (tr.index.buckets != nullptr) {
            if ((reinterpret_cast<uintptr_t>(tr.index.buckets) & 63) != 0 || tr.index.n_buckets != index_buckets(tr.run.n) || tr.run.n >= 0xFFFFFFFFull)
                return LSM_ERR_BAD_ARG;
            if (tr.run.n == 0) d.index = nullptr;
        }
        d.bloom = static_cast<const uint4*>(tr.bloom.blocks);
        d.bloom_blocks = tr.bloom.blocks ? (uint32_t)tr.bloom.n_blocks : 0;
        if (tr.bloom.blocks != nullptr &&
            (tr.bloom.n_blocks == 0 || tr.bloom.n_blocks >= (1ull << 32) || (reinterpret_cast<uintptr_t>(tr.bloom.blocks) & 15) != 0))
            return LSM_ERR_BAD_ARG;
        if (tr.run.n > 0) {
            if (tr.run.entries == nullptr || tr.fence.keys == nullptr) return LSM_ERR_NULL;
            if (tr.fence.stride == 0 || tr.fence.n != (tr.run.n + tr.fence.stride - 1) / tr.fence.stride) return LSM_ERR_BAD_ARG;
            if (tr.fence.n >= (1ull << 31)) return LSM_ERR_BAD_ARG;
            if ((reinterpret_cast<uintptr_t>(tr.run.entries) & 63) != 0 || (reinterpret_cast<uintptr_t>(tr.fence.keys) & 15) != 0)
                return LSM_ERR_BAD_ARG;
        } else {
            d.stride = 1;  // an empty run has no fences and is never searched
        }
    }
    tt.n_runs = tree->n_runs;
    for (uint32_t r = tree->n_runs; r < LSM_MAX_RUNS; r++) tt.run[r] = TreeRun{nullptr, nullptr, 0, nullptr, 1, 0, nullptr};
    return LSM_OK;
}

// Workgroups for n_req requests (one wave each): at most four per compute unit, each striding over the requests.
static int probe_grid(uint32_t n_req, uint32_t& blocks) {
    int device = 0, cus = 0;
    if (hipGetDevice(&device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || cus <= 0)
        return LSM_ERR_HIP;
    const uint32_t per_block = lsm::kProbeThreads / lsm::kWave;
    blocks = (n_req + per_block - 1) / per_block;
    if (blocks > (uint32_t)cus * 4) blocks = (uint32_t)cus * 4;
    return LSM_OK;
}

extern "C" int lsm_probe(const lsm_queries_t* queries, const lsm_tree_t* tree, const lsm_hits_t* out_hits, void* stream) {
    using namespace lsm;
    if (queries == nullptr || tree == nullptr || out_hits == nullptr) return LSM_ERR_NULL;
    if (queries->max_blocks == 0 || queries->max_blocks > LSM_MAX_BLOCKS || tree->n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    if (queries->n_req == 0) return LSM_OK;
    if (queries->keys == nullptr || queries->n_blocks == nullptr || out_hits->hit_len == nullptr || out_hits->hits == nullptr)
        return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(queries->keys) & 15) != 0 || (reinterpret_cast<uintptr_t>(out_hits->hits) & 15) != 0)
        return LSM_ERR_BAD_ARG;
    TreeTable tt;
    uint32_t blocks = 0;
    int rc = make_tree_table(tree, tt);
    if (rc == LSM_OK) rc = probe_grid(queries->n_req, blocks);
    if (rc != LSM_OK) return rc;
    if (all_indexed(tt))
        hipLaunchKernelGGL(probe_kernel<false>, dim3(blocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), tt, queries->keys,
                           queries->n_blocks, queries->n_req, queries->max_blocks, out_hits->hit_len, out_hits->hits);
    else
        hipLaunchKernelGGL(probe_kernel<true>, dim3(blocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), tt, queries->keys,
                           queries->n_blocks, queries->n_req, queries->max_blocks, out_hits->hit_len, out_hits->hits);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

extern "C" int lsm_probe_length(const lsm_queries_t* queries, const lsm_tree_t* tree, uint32_t* hit_len, void* stream) {
    using namespace lsm;
    if (queries == nullptr || tree == nullptr) return LSM_ERR_NULL;
    if (queries->max_blocks == 0 || queries->max_blocks > LSM_MAX_BLOCKS || tree->n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    if (queries->n_req == 0) return LSM_OK;
    if (queries->keys == nullptr || queries->n_blocks == nullptr || hit_len == nullptr) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(queries->keys) & 15) != 0) return LSM_ERR_BAD_ARG;
    TreeTable tt;
    uint32_t blocks = 0;
    int rc = make_tree_table(tree, tt);
    if (rc == LSM_OK) rc = probe_grid(queries->n_req, blocks);
    if (rc != LSM_OK) return rc;
    if (all_indexed(tt))
        hipLaunchKernelGGL(probe_length_kernel<false>, dim3(blocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), tt, queries->keys,
                           queries->n_blocks, queries->n_req, queries->max_blocks, hit_len);
    else
        hipLaunchKernelGGL(probe_length_kernel<true>, dim3(blocks), dim3(kProbeThreads), 0, static_cast<hipStream_t>(stream), tt, queries->keys,
                           queries->n_blocks, queries->n_req, queries->max_blocks, hit_len);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

extern "C" int lsm_range_bounds(const lsm_tree_t* tree, const uint8_t* lo_key, const uint8_t* hi_key, uint64_t* bounds_out, void* stream) {
    using namespace lsm;
    if (tree == nullptr || lo_key == nullptr || hi_key == nullptr) return LSM_ERR_NULL;
    if (tree->n_runs == 0) return LSM_OK;
    if (bounds_out == nullptr) return LSM_ERR_NULL;
    TreeTable tt;
    const int rc = make_tree_table(tree, tt);
    if (rc != LSM_OK) return rc;
    Key k[2];
    const uint8_t* src[2] = {lo_key, hi_key};
    for (int b = 0; b < 2; b++)
        for (int w = 0; w < 4; w++) {
            uint64_t v = 0;
            for (int i = 0; i < 8; i++) v = (v << 8) | src[b][8 * w + i];  // big-endian words: numeric order = byte order
            k[b].w[w] = v;
        }
    hipLaunchKernelGGL(range_bounds_kernel, dim3(1), dim3(2 * LSM_MAX_RUNS), 0, static_cast<hipStream_t>(stream), tt, k[0], k[1], bounds_out);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
