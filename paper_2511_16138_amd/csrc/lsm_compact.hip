// lsm_compact: single-pass k-way merge of sorted runs (paper section 2.2, compaction).
//
// Three kernels on one stream:
//   init_kernel       clears the per-call scratch (ticket, tile status words) and writes the
//                     first and last partition rows.
//   partition_kernel  one wave per interior tile boundary: multi-sequence selection over the
//                     k runs.  For target rank r it finds the key x with the largest
//                     L(x) = sum_j |{e in run j : e.key < x}| that is still <= r, and stores
//                     the k lower bounds.  Boundaries are therefore key-aligned (all versions
//                     of a key fall into the same tile) and tile sizes are within k of the
//                     nominal size.
//   merge_kernel      one workgroup per tile: stage the tile's entries in LDS, merge the k
//                     sorted pieces by ceil(log2 k) rounds of stable two-way merge-path merges
//                     over 16-bit indices, mark the newest version of every key, drop the rest
//                     (and winning tombstones when the output is the last level), compact the
//                     survivors with a block prefix sum, obtain the tile's output offset by a
//                     decoupled look-back over the tile status words, and copy the survivors
//                     out with coalesced 16-byte stores.  Every input byte is read once and
//                     every surviving byte written once.
#include <hip/hip_runtime.h>

#include "lsm_common.h"

namespace lsm {

constexpr int kMergeThreads = 256;
constexpr int kMergeItems = 4;
constexpr int kTileCap = kMergeThreads * kMergeItems;  // entries staged in LDS per tile
constexpr int kTileNominal = kTileCap - LSM_MAX_RUNS;  // boundary spacing in merged rank
constexpr uint32_t kSpinLimit = 1u << 22;              // polls of one look-back window before giving up

// Tile status word: top two bits = state, low 62 bits = value.
constexpr uint64_t kStEmpty = 0, kStAggregate = 1, kStPrefix = 2, kStFailed = 3;
constexpr int kStShift = 62;
constexpr uint64_t kStValueMask = (1ull << kStShift) - 1;

struct Header {  // first 256 bytes of the workspace
    uint32_t ticket;
    uint32_t validate_status;
    uint64_t reserved[31];
};
static_assert(sizeof(Header) == 256, "header is 256 bytes");

struct Workspace {
    Header* hdr;
    uint64_t* status;  // [n_tiles]
    uint64_t* splits;  // [(n_tiles + 1) * k]
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

__global__ void init_kernel(RunTable rt, Workspace ws, uint64_t n_tiles, uint64_t* n_out) {
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    if (i == 0) {
        ws.hdr->ticket = 0;
        ws.hdr->validate_status = 0;
        if (n_tiles == 0) *n_out = 0;
    }
    for (uint64_t t = i; t < n_tiles; t += stride) ws.status[t] = 0;
    if (i < rt.k) {
        ws.splits[i] = 0;
        ws.splits[n_tiles * rt.k + i] = rt.n[i];
    }
}

// ---------------------------------------------------------------------------------------
// Partition: lane j of a wave owns run j.  Candidates for x are the entries still inside
// [lo_j, hi_j) of every run; each step takes the middle entry of the widest range as pivot,
// every lane finds the pivot's lower bound in its own range, and the sum decides which side
// of the pivot survives.  The pivot itself always leaves its range, so the loop ends.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) partition_kernel(RunTable rt, Workspace ws, uint64_t n_tiles) {
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t b = (uint64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave + 1;  // boundary 1..n_tiles-1
    if (b >= n_tiles) return;  // whole wave leaves together
    const uint64_t r = b * (uint64_t)kTileNominal;
    const bool own = lane < (int)rt.k;
    const lsm_entry_t* run = own ? rt.ptr[lane] : nullptr;
    uint64_t lo = 0, hi = own ? rt.n[lane] : 0, best = 0;
    for (;;) {
        uint64_t width = hi - lo;
        uint64_t widest = wave_max_u64((width << 6) | (uint64_t)lane);
        if ((widest >> 6) == 0) break;
        int src = (int)(widest & 63);
        uint64_t mid = lo + (width >> 1);
        Key pivot = {{0, 0, 0, 0}};
        if (lane == src) pivot = load_key(run + mid);
        for (int w = 0; w < 4; w++) pivot.w[w] = __shfl(pivot.w[w], src, kWave);
        uint64_t lb = lo, ub = lo;
        if (own) {
            lb = lower_bound_run(run, lo, hi, pivot);
            ub = lb;
            if (lb < hi && key_equal(load_key(run + lb), pivot)) ub = lb + 1;
        }
        uint64_t total = wave_sum_u64(own ? lb : 0);
        // on sorted input the pivot's own lane has lb == mid; the clamps only matter for
        // inputs that break the precondition, where they still halve the widest range
        if (total <= r) {
            best = lb;
            lo = (lane == src && ub < mid + 1) ? mid + 1 : ub;
        } else {
            hi = (lane == src && lb > mid) ? mid : lb;
        }
    }
    if (own) ws.splits[b * rt.k + lane] = best;
}

// ---------------------------------------------------------------------------------------
// Tile merge.
// ---------------------------------------------------------------------------------------
struct MergeShared {
    uint4 ent[kTileCap][4];      // staged entries, 64 bytes each
    uint16_t ord[2][kTileCap];   // ping-pong index lists; later ord[x] = survivor list
    uint8_t same[kTileCap + 1];  // same[i] = key at merged position i equals key at i-1
    uint32_t seg[LSM_MAX_RUNS + 1];  // start of each run's piece in tile-local index space
    uint64_t lo[LSM_MAX_RUNS];       // first entry of each run's piece
    uint32_t wave_count[kMergeThreads / kWave];
    uint32_t tile;
    uint32_t n;
    uint64_t base;
    uint32_t failed;
};

__device__ __forceinline__ Key lds_key(const MergeShared& s, uint32_t e) { return key_from_raw(s.ent[e][0], s.ent[e][1]); }
__device__ __forceinline__ uint64_t lds_seqno(const MergeShared& s, uint32_t e) {
    uint4 v = s.ent[e][2];
    return ((uint64_t)v.y << 32) | v.x;
}
__device__ __forceinline__ uint32_t lds_type(const MergeShared& s, uint32_t e) { return s.ent[e][2].z & 0xFF; }

// Publish this tile's survivor count and return the number of survivors in all earlier tiles
// (decoupled look-back).  Called by wave 0 only, all 64 lanes.  Tiles take their numbers from
// an atomic ticket, so every earlier tile has already started and will publish; the wait is
// bounded anyway, and a tile that gives up publishes kStFailed, which propagates forward.
__device__ uint64_t lookback(uint64_t* status, uint64_t tile, uint64_t count, bool self_failed, bool* failed) {
    const int lane = threadIdx.x & (kWave - 1);
    *failed = self_failed;
    if (self_failed) {
        if (lane == 0) __hip_atomic_store(&status[tile], kStFailed << kStShift, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return 0;
    }
    if (tile == 0) {
        if (lane == 0) __hip_atomic_store(&status[0], (kStPrefix << kStShift) | count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return 0;
    }
    if (lane == 0) __hip_atomic_store(&status[tile], (kStAggregate << kStShift) | count, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    uint64_t base = 0;
    int64_t top = (int64_t)tile - 1;  // lane l looks at tile top - l
    bool bad = false;
    for (;;) {
        int64_t t = top - lane;
        uint64_t st = kStPrefix << kStShift;  // tiles before tile 0: an empty prefix
        uint32_t spins = 0;
        for (;;) {
            if (t >= 0) st = __hip_atomic_load(&status[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            bool ready = (st >> kStShift) != kStEmpty;
            if (__ballot(!ready) == 0) break;
            if (++spins > kSpinLimit) {
                bad = true;
                break;
            }
            __builtin_amdgcn_s_sleep(2);
        }
        if (bad) break;
        uint64_t state = st >> kStShift;
        if (__ballot(state == kStFailed) != 0) {
            bad = true;
            break;
        }
        uint64_t pmask = __ballot(state == kStPrefix);
        int first = pmask ? __ffsll((unsigned long long)pmask) - 1 : kWave - 1;  // nearest tile with a full prefix
        base += wave_sum_u64(lane <= first ? (st & kStValueMask) : 0);
        if (pmask) break;
        top -= kWave;
    }
    *failed = bad;
    uint64_t word = bad ? (kStFailed << kStShift) : ((kStPrefix << kStShift) | (base + count));
    if (lane == 0) __hip_atomic_store(&status[tile], word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return base;
}

__global__ void __launch_bounds__(kMergeThreads) merge_kernel(RunTable rt, Workspace ws, uint64_t n_tiles, uint32_t flags,
                                                               lsm_entry_t* out, uint64_t* n_out) {
    __shared__ MergeShared s;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const uint32_t k = rt.k;

    // ---- tile number (ticket order = output order) and its k pieces
    if (tid == 0) s.tile = atomicAdd(&ws.hdr->ticket, 1u);
    __syncthreads();
    const uint64_t tile = s.tile;
    if (tile >= n_tiles) return;  // cannot happen: the grid has exactly n_tiles workgroups
    if (tid < (int)k) {
        uint64_t a = ws.splits[tile * k + tid], b = ws.splits[(tile + 1) * k + tid];
        s.lo[tid] = a;
        s.seg[tid + 1] = (uint32_t)(b >= a ? b - a : 0);
    }
    __syncthreads();
    if (tid == 0) {
        uint32_t acc = 0;
        s.seg[0] = 0;
        bool ok = true;
        for (uint32_t j = 0; j < k; j++) {
            uint32_t len = s.seg[j + 1];
            if (len > (uint32_t)kTileCap || s.lo[j] + len > rt.n[j]) {
                ok = false;
                len = 0;
            }
            acc += len;
            s.seg[j + 1] = acc;
        }
        if (acc > (uint32_t)kTileCap) ok = false;
        s.n = ok ? acc : 0;
        s.failed = ok ? 0 : 1;
    }
    __syncthreads();
    const uint32_t n = s.n;

    // ---- stage the tile in LDS: 4 lanes per entry, 16 bytes each, coalesced
    for (uint32_t c = tid; c < n * 4; c += kMergeThreads) {
        uint32_t e = c >> 2, part = c & 3;
        uint32_t j = 0;
        for (uint32_t step = 32; step > 0; step >>= 1)  // last j with seg[j] <= e
            if (j + step < k && s.seg[j + step] <= e) j += step;
        while (j + 1 < k && s.seg[j + 1] <= e) j++;  // skip empty pieces that start at the same offset
        const uint4* src = reinterpret_cast<const uint4*>(rt.ptr[j] + s.lo[j] + (e - s.seg[j]));
        s.ent[e][part] = src[part];
    }
    for (uint32_t e = tid; e < n; e += kMergeThreads) s.ord[0][e] = (uint16_t)e;
    __syncthreads();

    // ---- merge rounds: lists of `width` runs each are merged pairwise, stable (left list first)
    int cur = 0;
    for (uint32_t width = 1; width < k; width <<= 1) {
        const uint16_t* in = s.ord[cur];
        uint16_t* dst = s.ord[cur ^ 1];
        uint32_t o = tid * kMergeItems;
        const uint32_t o_end = min(o + (uint32_t)kMergeItems, n);
        while (o < o_end) {
            // the pair of lists whose output range contains position o
            uint32_t j = 0;
            for (uint32_t step = 32; step > 0; step >>= 1)
                if (j + step < k && s.seg[j + step] <= o) j += step;
            while (j + 1 < k && s.seg[j + 1] <= o) j++;
            uint32_t pair = j / (2 * width);
            uint32_t ra = pair * 2 * width, rb = min(ra + width, k), rc = min(ra + 2 * width, k);
            uint32_t sa = s.seg[ra], sb = s.seg[rb], sc = s.seg[rc];
            uint32_t len_a = sb - sa, len_b = sc - sb;
            uint32_t stop = min(o_end, sc);
            // co-rank of diagonal d: how many of the first d outputs come from the left list
            uint32_t d = o - sa;
            uint32_t lo = d > len_b ? d - len_b : 0, hi = min(d, len_a);
            while (lo < hi) {
                uint32_t mid = (lo + hi) >> 1;
                Key ka = lds_key(s, in[sa + mid]);
                Key kb = lds_key(s, in[sb + (d - 1 - mid)]);
                if (key_less_equal(ka, kb)) lo = mid + 1;
                else hi = mid;
            }
            uint32_t a = lo, b = d - lo;
            uint32_t ia = a < len_a ? in[sa + a] : 0, ib = b < len_b ? in[sb + b] : 0;
            Key ka = lds_key(s, ia), kb = lds_key(s, ib);
            for (; o < stop; o++) {
                bool take_a = b >= len_b || (a < len_a && key_less_equal(ka, kb));
                dst[o] = (uint16_t)(take_a ? ia : ib);
                if (take_a) {
                    a++;
                    ia = a < len_a ? in[sa + a] : 0;
                    ka = lds_key(s, ia);
                } else {
                    b++;
                    ib = b < len_b ? in[sb + b] : 0;
                    kb = lds_key(s, ib);
                }
            }
        }
        __syncthreads();
        cur ^= 1;
    }
    const uint16_t* ord = s.ord[cur];
    uint16_t* surv = s.ord[cur ^ 1];

    // ---- same[i]: merged position i repeats the key of position i-1
    {
        uint32_t o = tid * kMergeItems;
        const uint32_t o_end = min(o + (uint32_t)kMergeItems, n);
        if (o < o_end) {
            Key prev = lds_key(s, ord[o > 0 ? o - 1 : 0]);
            for (; o < o_end; o++) {
                Key kk = lds_key(s, ord[o]);
                s.same[o] = (o > 0 && key_equal(prev, kk)) ? 1 : 0;
                prev = kk;
            }
        }
        if (tid == 0) s.same[n] = 0;
    }
    __syncthreads();

    // ---- survivors: newest version of each key (largest seqno, ties to the earlier = lower run),
    //      minus winning tombstones when the output is the last level
    uint32_t keep_mask = 0, my_count = 0;
    {
        const uint32_t o0 = tid * kMergeItems;
        for (uint32_t i = 0; i < (uint32_t)kMergeItems; i++) {
            uint32_t o = o0 + i;
            if (o >= n) break;
            uint32_t e = ord[o];
            uint64_t seq = lds_seqno(s, e);
            bool win = true;
            for (uint32_t p = o; s.same[p]; p--)  // earlier members of the group (same[0] is 0)
                if (lds_seqno(s, ord[p - 1]) >= seq) win = false;
            for (uint32_t p = o + 1; s.same[p]; p++)  // later members (same[n] is 0)
                if (lds_seqno(s, ord[p]) > seq) win = false;
            if (win && (flags & LSM_BOTTOMMOST) && lds_type(s, e) == LSM_TOMBSTONE) win = false;
            if (win) {
                keep_mask |= 1u << i;
                my_count++;
            }
        }
    }
    // block-wide exclusive prefix of my_count
    uint32_t incl = my_count;
    for (int off = 1; off < kWave; off <<= 1) {
        uint32_t v = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += v;
    }
    if (lane == kWave - 1) s.wave_count[wave] = incl;
    __syncthreads();
    uint32_t wave_base = 0, total = 0;
    for (int w = 0; w < kMergeThreads / kWave; w++) {
        uint32_t c = s.wave_count[w];
        if (w < wave) wave_base += c;
        total += c;
    }
    {
        uint32_t pos = wave_base + incl - my_count;
        const uint32_t o0 = tid * kMergeItems;
        for (uint32_t i = 0; i < (uint32_t)kMergeItems; i++)
            if (keep_mask & (1u << i)) surv[pos++] = ord[o0 + i];
    }

    // ---- output offset of this tile
    if (wave == 0) {
        bool failed;
        uint64_t base = lookback(ws.status, tile, total, s.failed != 0, &failed);
        if (lane == 0) {
            s.base = base;
            if (failed) s.failed = 1;
        }
    }
    __syncthreads();
    const bool failed = s.failed != 0;
    const uint64_t base = s.base;
    if (tile == n_tiles - 1 && tid == 0) *n_out = failed ? ~0ull : base + total;
    if (failed) return;

    // ---- copy survivors out: 4 lanes per entry, 16 bytes each
    uint4* dst = reinterpret_cast<uint4*>(out + base);
    for (uint32_t c = tid; c < total * 4; c += kMergeThreads) dst[c] = s.ent[surv[c >> 2]][c & 3];
}

// ---------------------------------------------------------------------------------------
// Optional input check (LSM_VALIDATE): every run strictly ascending, type bytes valid.
// ---------------------------------------------------------------------------------------
__global__ void validate_kernel(RunTable rt, Workspace ws) {
    const uint32_t j = blockIdx.y;
    const lsm_entry_t* run = rt.ptr[j];
    const uint64_t n = rt.n[j];
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    uint32_t bad = 0;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        if (run[i].type > LSM_TOMBSTONE) bad |= 2;
        if (i + 1 < n && !key_less(load_key(run + i), load_key(run + i + 1))) bad |= 1;
    }
    if (bad) atomicOr(&ws.hdr->validate_status, bad);
}

static Workspace carve(void* base, uint64_t n_tiles, uint32_t k) {
    char* p = static_cast<char*>(base);
    Workspace ws;
    ws.hdr = reinterpret_cast<Header*>(p);
    ws.status = reinterpret_cast<uint64_t*>(p + sizeof(Header));
    ws.splits = reinterpret_cast<uint64_t*>(p + sizeof(Header) + align256(n_tiles * sizeof(uint64_t)));
    (void)k;
    return ws;
}

static uint64_t tiles_for(uint64_t total) { return (total + kTileNominal - 1) / kTileNominal; }

}  // namespace lsm

extern "C" size_t lsm_compact_workspace_bytes(const uint64_t* run_lens, uint32_t n_runs) {
    if (run_lens == nullptr || n_runs == 0 || n_runs > LSM_MAX_RUNS) return 0;
    uint64_t total = 0;
    for (uint32_t j = 0; j < n_runs; j++) total += run_lens[j];
    uint64_t n_tiles = lsm::tiles_for(total);
    return sizeof(lsm::Header) + lsm::align256(n_tiles * sizeof(uint64_t)) +
           lsm::align256((n_tiles + 1) * (uint64_t)n_runs * sizeof(uint64_t));
}

extern "C" int lsm_compact(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                           size_t workspace_bytes, void* stream) {
    return lsm_compact_timed(runs, n_runs, flags, out, workspace, workspace_bytes, stream, nullptr);
}

extern "C" int lsm_compact_timed(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                                 size_t workspace_bytes, void* stream_v, const lsm_compact_events_t* ev) {
    using namespace lsm;
    if (runs == nullptr || out == nullptr || out->n_out == nullptr) return LSM_ERR_NULL;
    if (n_runs == 0 || n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    RunTable rt;
    rt.k = n_runs;
    uint64_t total = 0;
    for (uint32_t j = 0; j < LSM_MAX_RUNS; j++) {
        rt.ptr[j] = nullptr;
        rt.n[j] = 0;
    }
    for (uint32_t j = 0; j < n_runs; j++) {
        if (runs[j].n > 0 && runs[j].entries == nullptr) return LSM_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(runs[j].entries) & 63) != 0) return LSM_ERR_BAD_ARG;
        rt.ptr[j] = runs[j].entries;
        rt.n[j] = runs[j].n;
        total += runs[j].n;
    }
    if (total > 0 && out->entries == nullptr) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(out->entries) & 63) != 0) return LSM_ERR_BAD_ARG;
    if (out->capacity < total) return LSM_ERR_CAPACITY;
    uint64_t lens[LSM_MAX_RUNS];
    for (uint32_t j = 0; j < n_runs; j++) lens[j] = runs[j].n;
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 ||
        workspace_bytes < lsm_compact_workspace_bytes(lens, n_runs))
        return LSM_ERR_WORKSPACE;
    const uint64_t n_tiles = tiles_for(total);
    if (n_tiles >= (1ull << 31)) return LSM_ERR_BAD_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    Workspace ws = carve(workspace, n_tiles, n_runs);

    uint32_t init_blocks = (uint32_t)((n_tiles + 255) / 256);
    if (init_blocks == 0) init_blocks = 1;
    if (init_blocks > 1024) init_blocks = 1024;
    hipLaunchKernelGGL(init_kernel, dim3(init_blocks), dim3(256), 0, stream, rt, ws, n_tiles, out->n_out);

    if (flags & LSM_VALIDATE) {
        hipLaunchKernelGGL(validate_kernel, dim3(256, n_runs), dim3(256), 0, stream, rt, ws);
        uint32_t vs = 0;
        if (hipMemcpyAsync(&vs, &ws.hdr->validate_status, sizeof(vs), hipMemcpyDeviceToHost, stream) != hipSuccess)
            return LSM_ERR_HIP;
        if (hipStreamSynchronize(stream) != hipSuccess) return LSM_ERR_HIP;
        if (vs & 1) return LSM_ERR_UNSORTED;
        if (vs & 2) return LSM_ERR_BAD_ENTRY;
    }
    if (ev && ev->before_partition && hipEventRecord(static_cast<hipEvent_t>(ev->before_partition), stream) != hipSuccess)
        return LSM_ERR_HIP;
    if (n_tiles > 1) {
        uint32_t waves_per_block = 256 / kWave;
        uint32_t blocks = (uint32_t)((n_tiles - 1 + waves_per_block - 1) / waves_per_block);
        hipLaunchKernelGGL(partition_kernel, dim3(blocks), dim3(256), 0, stream, rt, ws, n_tiles);
    }
    if (ev && ev->before_merge && hipEventRecord(static_cast<hipEvent_t>(ev->before_merge), stream) != hipSuccess)
        return LSM_ERR_HIP;
    if (n_tiles > 0)
        hipLaunchKernelGGL(merge_kernel, dim3((uint32_t)n_tiles), dim3(kMergeThreads), 0, stream, rt, ws, n_tiles, flags,
                           out->entries, out->n_out);
    if (ev && ev->after_merge && hipEventRecord(static_cast<hipEvent_t>(ev->after_merge), stream) != hipSuccess)
        return LSM_ERR_HIP;
    if (hipGetLastError() != hipSuccess) return LSM_ERR_HIP;
    if (flags & LSM_VALIDATE) {
        uint64_t n = 0;
        if (hipMemcpyAsync(&n, out->n_out, sizeof(n), hipMemcpyDeviceToHost, stream) != hipSuccess) return LSM_ERR_HIP;
        if (hipStreamSynchronize(stream) != hipSuccess) return LSM_ERR_HIP;
        if (n == ~0ull) return LSM_ERR_INTERNAL;
    }
    return LSM_OK;
}
