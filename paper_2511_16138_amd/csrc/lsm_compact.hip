// lsm_compact: single-pass k-way merge of sorted runs (paper section 2.2, compaction).
//
// Kernels, on one stream:
//   init_kernel       clears the per-call scratch (tile status words) and writes the
//                     first and last partition rows (inputs of a few tiles: done by the
//                     partition launch instead).
//   partition         one group of lanes per interior tile boundary: multi-sequence selection
//                     over the k runs.  For target rank r it finds the key x with the largest
//                     L(x) = sum_j |{e in run j : e.key < x}| that is still <= r, and stores
//                     the k lower bounds.  Boundaries are therefore key-aligned (all versions
//                     of a key fall into the same tile) and tile sizes are within k of the
//                     nominal size.  Small inputs search the runs directly (partition_kernel);
//                     large ones first bracket every boundary on a copy of every 32nd key
//                     (sample_kernel, sample_coarse_kernel, sample_fine_kernel) and search the
//                     runs only inside the brackets (bracket_partition_kernel).
//   merge_kernel      one workgroup per tile: every thread loads its share of the tile's entries
//                     into registers, 16-byte surrogates (14 key bytes + index) are merged in LDS
//                     by ceil(log2 k) rounds of stable two-way merge-path merges, the newest
//                     version of every key is marked, the rest (and winning tombstones when the
//                     output is the last level) dropped, survivors are counted with a block
//                     prefix sum, the tile's output offset comes from a decoupled look-back over
//                     the tile status words, and the survivors leave through an LDS stage with
//                     contiguous 16-byte stores.  Every input byte is read once and every
//                     surviving byte written once.
#include <hip/hip_runtime.h>

#include <string.h>

#include <mutex>

#include "lsm_common.h"

namespace lsm {

constexpr int kMergeThreads = 512;
constexpr int kMergeItems = 4;
constexpr int kTileCap = kMergeThreads * kMergeItems;  // entries per tile
constexpr int kRoundItems = 4;                         // outputs per thread in a merge round
// Boundary spacing in merged rank for k runs: a tile is at most k - 1 entries longer than this (keys are unique
// inside a run, so the boundary key's rank is less than k short of its target), which is the tile capacity.
__host__ __device__ inline uint64_t tile_nominal(uint32_t k) { return (uint64_t)kTileCap - k; }
constexpr uint64_t kCoarseStride = 16;                 // every 16th boundary is searched over whole sequences first
constexpr uint64_t kSampleStride = 32;                 // one key in 32 is copied for the sampled partition
constexpr uint64_t kShortRunsTotal = 262144;           // inputs of at most this many entries (16 MiB) are searched as cached data
constexpr uint64_t kSampledMinTiles = 2048;            // inputs of fewer tiles search the runs directly (measured crossover)
constexpr uint32_t kSpinLimit = 1u << 22;              // polls of one look-back window before giving up

// Tile status word: top two bits = state, low 62 bits = value.
constexpr uint64_t kStEmpty = 0, kStAggregate = 1, kStPrefix = 2, kStFailed = 3;
constexpr int kStShift = 62;
constexpr uint64_t kStValueMask = (1ull << kStShift) - 1;

struct Header {  // first 256 bytes of the workspace
    uint32_t unused;
    uint32_t validate_status;
    uint64_t reserved[31];
};
static_assert(kRoundItems == 4, "the register merge network is written for four outputs");
static_assert(sizeof(Header) == 256, "header is 256 bytes");

// A bare 32-byte key: one sample of a run.
struct SampleKey {
    uint4 q[2];
};

struct SampleTable {
    SampleKey* ptr[LSM_MAX_RUNS];
    uint64_t m[LSM_MAX_RUNS];  // samples of run j = ceil(n[j] / kSampleStride)
};

struct Workspace {
    Header* hdr;
    uint64_t* status;   // [n_tiles]
    uint64_t* splits;   // [(n_tiles + 1) * k]
    uint64_t* ycoarse;  // [(n_coarse + 2) * k]   sample-space splits of every kCoarseStride-th boundary
    uint64_t* ywin;     // [2 * (n_tiles - 1) * k] sample-space brackets of every boundary
    SampleTable st;
};

__host__ __device__ inline size_t align256(size_t x) { return (x + 255) & ~size_t(255); }

__global__ void init_kernel(RunTable rt, Workspace ws, uint64_t n_tiles, uint64_t n_coarse, uint64_t* n_out) {
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    if (i == 0) {
        ws.hdr->validate_status = 0;
        if (n_tiles == 0) *n_out = 0;
    }
    for (uint64_t t = i; t < n_tiles; t += stride) ws.status[t] = 0;
    if (i < rt.k) {
        ws.splits[i] = 0;
        ws.splits[n_tiles * rt.k + i] = run_len(rt, (uint32_t)i);
        ws.ycoarse[i] = 0;
        ws.ycoarse[(n_coarse + 1) * rt.k + i] = ws.st.m[i];
    }
}

// ---------------------------------------------------------------------------------------
// Partition: a group of G lanes (G = smallest power of two >= k) works on one selection
// problem, lane j of the group owns sequence j, and a wave handles 64/G problems at once.
// For a target rank r the problem is: among the records still inside [lo_j, hi_j) of every
// sequence, find the key x with the largest L(x) = sum_j |{e in sequence j : e.key < x}| that
// is still <= r, and return the k lower bounds of x.  Each step takes a record of the widest
// range as pivot, every lane finds the pivot's lower bound in its own range, and the sum over
// the group decides which side of the pivot survives.  The pivot always leaves its range and
// the widest range at least halves every third step, so the loop ends after at most
// 3 * k * log2(longest sequence) steps whatever the input.
//
// The ranges need not be cuts of one key: it is enough that lo_j <= (the answer's lower bound
// in j) <= hi_j and that the answer itself lies inside its own sequence's range.  Lower bounds
// are then clamped into the ranges, which never changes on which side of r a sum falls.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t group_sum_u64(uint64_t v, int group) {
    for (int off = group >> 1; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ uint64_t group_max_u64(uint64_t v, int group) {
    for (int off = group >> 1; off > 0; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

constexpr int kTailKeys = 4;        // ranges this short are finished from registers
constexpr int kTailKeysCached = 2;  // the same for searches on the cached sample arrays

// One step's bookkeeping once every lane has its lower bound lb (and whether the record there equals the pivot).
__device__ __forceinline__ void select_update(uint64_t& lo, uint64_t& hi, uint64_t& best, const uint64_t lb, const bool eq,
                                              const uint64_t mid, const bool is_src, const bool active, const bool own,
                                              const uint64_t r, const int group) {
    const uint64_t total = group_sum_u64(own ? lb : 0, group);
    if (!active) return;
    // on sorted input the pivot's own lane has lb == mid; the clamps only matter for inputs that
    // break the precondition, where they still shrink the widest range
    const uint64_t ub = lb + (eq ? 1 : 0);
    if (total <= r) {
        best = lb;
        lo = (is_src && ub < mid + 1) ? mid + 1 : ub;
    } else {
        hi = (is_src && lb > mid) ? mid : lb;
    }
}

template <bool kCached, typename E>
__device__ __forceinline__ uint64_t select_split(const E* run, uint64_t lo, uint64_t hi, const uint64_t r, const bool own,
                                                 const int member, const int group, const int group_base) {
    uint64_t best = lo;
    // on the cached sample arrays a shorter tail keeps the kernel at 64 registers (8 waves per SIMD), worth more there
    constexpr int kTail = kCached ? kTailKeysCached : kTailKeys;
    // phase 1: pivots and lower bounds from memory, until every range of the group is at most kTail long
    for (uint32_t iter = 0;; iter++) {
        const uint64_t width = hi - lo;
        const uint64_t widest = group_max_u64((width << 6) | (uint64_t)member, group);
        const bool active = (widest >> 6) > (uint64_t)kTail;
        if (__ballot(active) == 0) break;
        const int src = (int)(widest & 63);
        // bisection steps take the roundest position of the middle quarter when the records are in HBM
        // (a position other searches read too), the plain middle when they are cached
        uint64_t mid = lo + (width >> 1);
        if (!kCached && width) mid = tree_mid(lo + ((3 * width) >> 3), lo + ((5 * width) >> 3) + 1);
        if (iter % 3 != 2) {
            // interpolation steps: the candidates are the merged ranks [sum lo, sum hi); aim the pivot at
            // the same fraction of the widest range as a target rank is of that interval.  The target
            // is r minus, then r plus, a margin of the order of the estimate's standard deviation (the
            // square root of the interval: one such on the cached sample arrays, a quarter where every probe
            // is an HBM access and a missed bracket costs less than a wide one - both measured), so that two
            // steps bracket x from both sides.  Every third step is a bisection step, which keeps the worst
            // case logarithmic.
            const uint64_t rank_lo = group_sum_u64(own ? lo : 0, group), rank_hi = group_sum_u64(own ? hi : 0, group);
            uint64_t span = rank_hi - rank_lo, ahead = r > rank_lo ? r - rank_lo : 0;
            const uint64_t margin = span ? (1ull << ((64 - __builtin_clzll(span)) >> 1)) >> (kCached ? 0 : 2) : 0;
            if (iter % 3 == 0) ahead = ahead > margin ? ahead - margin : 0;
            else ahead += margin;
            if (ahead > span) ahead = span;
            const int shift = span >> 31 ? 64 - __builtin_clzll(span) - 31 : 0;
            span >>= shift;
            ahead >>= shift;
            uint64_t frac = span ? (ahead << 32) / span : 0;  // 32.32 fixed point in [0, 1]
            if (frac > 0xFFFFFFFFull) frac = 0xFFFFFFFFull;
            if (rank_hi - rank_lo >= 256 && width > 0 && width <= 0xFFFFFFFFull) {  // few candidates left: plain bisection
                mid = lo + ((width * frac) >> 32);
                if (mid >= hi) mid = hi - 1;
                // the roundest position within 1/16 of the range around the aim: likely read before, or again later
                const uint64_t slack = width >> 4;
                if (!kCached) mid = tree_mid(mid - lo > slack ? mid - slack : lo, hi - mid > slack + 1 ? mid + slack + 1 : hi);
            }
        }
        Key pivot = {{0, 0, 0, 0}};
        if (active && member == src) pivot = load_key(run + mid);
        for (int w = 0; w < 4; w++) pivot.w[w] = __shfl(pivot.w[w], group_base + src, kWave);
        uint64_t lb = lo;
        bool eq = false;
        if (own && active) lb = kCached ? lower_bound_eq4(run, lo, hi, pivot, eq) : lower_bound_eq(run, lo, hi, pivot, eq);
        select_update(lo, hi, best, lb, eq, mid, member == src, active, own, r, group);
    }
    // phase 2: the same steps on the at most kTail keys per range that are left, held in registers
    const uint64_t base = lo;
    const int cnt = (int)(hi - lo);  // <= kTail
    Key kk[kTail];
    for (int i = 0; i < kTail; i++) kk[i] = i < cnt ? load_key(run + base + i) : Key{{0, 0, 0, 0}};
    for (;;) {
        const uint64_t width = hi - lo;
        const uint64_t widest = group_max_u64((width << 6) | (uint64_t)member, group);
        const bool active = (widest >> 6) != 0;
        if (__ballot(active) == 0) break;
        const int src = (int)(widest & 63);
        const uint64_t mid = lo + (width >> 1);
        const int at = (int)(mid - base);
        Key pivot = kk[0];
        for (int i = 1; i < kTail; i++)
            if (at == i) pivot = kk[i];
        for (int w = 0; w < 4; w++) pivot.w[w] = __shfl(pivot.w[w], group_base + src, kWave);
        uint64_t lb = base;
        for (int i = 0; i < kTail; i++) lb += (i < cnt && key_less(kk[i], pivot)) ? 1 : 0;
        lb = lb < lo ? lo : (lb > hi ? hi : lb);
        bool eq = false;
        for (int i = 0; i < kTail; i++) eq = eq || (lb < hi && lb == base + i && key_equal(kk[i], pivot));
        select_update(lo, hi, best, lb, eq, mid, member == src, active, own, r, group);
    }
    return best;
}

// Two runs: the boundary of merged rank r by bisection on the merge path - how many entries of `a` are among the first r
// of the merged order (equal keys: a's first) - with two independent reads per step, then moved back by one entry when
// the two versions of a key would fall on either side of it.  Same result as select_split (the lower bounds of the key x
// with the largest L(x) <= r) in log2 of the shorter run's length dependent steps instead of a pivoting selection.
__device__ __forceinline__ void split_two(const lsm_entry_t* a, const uint64_t na, const lsm_entry_t* b, const uint64_t nb, const uint64_t r,
                                          uint64_t& ia, uint64_t& ib) {
    const uint64_t d = r < na + nb ? r : na + nb;
    uint64_t lo = d > nb ? d - nb : 0, hi = d < na ? d : na;  // the count lies in [lo, hi]
    while (lo < hi) {
        const uint64_t mid = lo + (hi - lo + 1) / 2;  // lo < mid <= hi, so d - mid < nb
        // mid entries of a fit among the first d iff a[mid - 1] does not come after b[d - mid]
        if (key_less_equal(load_key(a + mid - 1), load_key(b + (d - mid)))) lo = mid;
        else hi = mid - 1;
    }
    ia = lo;
    ib = d - lo;
    // a's version of a key just before the boundary and b's just after it: the key starts one entry earlier
    if (ia > 0 && ib < nb && key_equal(load_key(a + ia - 1), load_key(b + ib))) ia--;
}

// Lane bookkeeping shared by the partition kernels: which problem and which sequence a lane has.
struct GroupLane {
    int member, group_base;
    uint64_t slot;
};
__device__ __forceinline__ GroupLane group_lane(int group) {
    const int lane = threadIdx.x & (kWave - 1);
    GroupLane g;
    g.member = lane & (group - 1);
    g.group_base = lane - g.member;
    const uint64_t wave_id = (uint64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    g.slot = wave_id * (uint64_t)(kWave / group) + (uint64_t)(lane / group);
    return g;
}

// Direct search over whole runs, for inputs of a few dozen tiles: one launch, one group per interior boundary.
// kInit: the launch also clears the tile status words and writes the first and last split rows, which saves the
// separate init launch (a small compaction is then two launches: this one and the merge).  kShort: the runs are
// short enough to stay in cache, where four-way search steps (half the dependent round trips) are the faster ones.
template <bool kInit, bool kShort>
__global__ void __launch_bounds__(256) partition_kernel(RunTable rt, Workspace ws, uint64_t n_tiles, int group) {
    if (kInit) {
        const uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (uint64_t)gridDim.x * blockDim.x;
        for (uint64_t t = i; t < n_tiles; t += stride) ws.status[t] = 0;
        if (i < rt.k) {
            ws.splits[i] = 0;
            ws.splits[n_tiles * rt.k + i] = run_len(rt, (uint32_t)i);
        }
    }
    const GroupLane g = group_lane(group);
    const uint64_t b = g.slot + 1;
    const bool own = b < n_tiles && g.member < (int)rt.k;
    if (rt.k == 2) {  // two runs (every merge of a leveled tree): the merge path is a plain bisection
        if (own && g.member == 0) {
            uint64_t ia, ib;
            split_two(rt.ptr[0], run_len(rt, 0), rt.ptr[1], run_len(rt, 1), b * tile_nominal(2), ia, ib);
            ws.splits[b * 2 + 0] = ia;
            ws.splits[b * 2 + 1] = ib;
        }
        return;
    }
    const lsm_entry_t* run = own ? rt.ptr[g.member] : nullptr;
    const uint64_t best = select_split<kShort>(run, 0, own ? run_len(rt, g.member) : 0, b * tile_nominal(rt.k), own, g.member, group, g.group_base);
    if (own) ws.splits[b * rt.k + g.member] = best;
}

// ---------------------------------------------------------------------------------------
// Sampled partition, for large inputs.  Searching the runs directly costs tens of scattered
// 64-byte reads per boundary and run, which is HBM traffic of the order of the merge itself.
// Instead every kSampleStride-th key of each run is copied into a compact array (1/64 of the
// input bytes: it stays in the last-level cache), the selection is done on the samples, and the
// runs themselves are only searched inside the few dozen entries the samples leave open.
//
// With s = kSampleStride, a key P that has y_j samples below it in run j has x_j entries below
// it with s * (y_j - 1) < x_j <= s * y_j, so for Y = sum y_j:  s * (Y - k) < L(P) <= s * Y.
//   lower bracket: the sample key with the largest Y <= floor(r / s) has L <= r, so it is <= x;
//   upper bracket: the sample key with the largest Y <= ceil(r / s) + 2k - 1 has, if a larger sample
//                  exists at all, Y >= ceil(r / s) + k and therefore L > r: it is > x.
// The answer's lower bound in run j then lies in [s * (ylo_j - 1) + 1, s * yhi_j] (clamped to the run).
// The sample-space problems are themselves solved coarse first: every kCoarseStride-th boundary
// over whole sample arrays, the rest between the coarse rows that enclose their targets.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) sample_kernel(RunTable rt, SampleTable st) {
    const uint32_t j = blockIdx.y;
    const uint4* src = reinterpret_cast<const uint4*>(rt.ptr[j]);
    uint4* dst = reinterpret_cast<uint4*>(st.ptr[j]);
    const uint64_t n16 = st.m[j] * 2, stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride)
        dst[i] = src[(i >> 1) * (kSampleStride * 4) + (i & 1)];  // 4 uint4 per entry; two lanes copy one key
}

__device__ __forceinline__ uint64_t sample_target(uint64_t b, int side, uint32_t k) {
    const uint64_t r = b * tile_nominal(k);
    return side ? (r + kSampleStride - 1) / kSampleStride + 2ull * k - 1 : r / kSampleStride;
}

// coarse rows: row c (1 <= c <= n_coarse) = lower bracket of boundary c * kCoarseStride over whole sample arrays
__global__ void __launch_bounds__(256) sample_coarse_kernel(Workspace ws, uint32_t k, uint64_t n_coarse, int group) {
    const GroupLane g = group_lane(group);
    const uint64_t c = g.slot + 1;
    const bool own = c <= n_coarse && g.member < (int)k;
    const SampleKey* run = own ? ws.st.ptr[g.member] : nullptr;
    const uint64_t best = select_split<true>(run, 0, own ? ws.st.m[g.member] : 0, sample_target(c * kCoarseStride, 0, k), own,
                                       g.member, group, g.group_base);
    if (own) ws.ycoarse[c * k + g.member] = best;
}

// problem p = 2 * (b - 1) + side for boundary b; targets of boundaries [c * stride, (c + 1) * stride) lie
// between those of coarse rows c and c + 2 (the upper bracket overshoots by 2k - 1 <= one coarse step)
__global__ void __launch_bounds__(256) sample_fine_kernel(Workspace ws, uint32_t k, uint64_t n_tiles, uint64_t n_coarse, int group) {
    const GroupLane g = group_lane(group);
    const uint64_t b = g.slot / 2 + 1;
    const int side = (int)(g.slot & 1);
    const bool own = b < n_tiles && g.member < (int)k;
    const SampleKey* run = own ? ws.st.ptr[g.member] : nullptr;
    uint64_t lo = 0, hi = 0;
    if (own) {
        const uint64_t c = b / kCoarseStride, above = c + 2 < n_coarse + 1 ? c + 2 : n_coarse + 1;
        lo = ws.ycoarse[c * k + g.member];
        hi = ws.ycoarse[above * k + g.member];
        if (hi > ws.st.m[g.member]) hi = ws.st.m[g.member];  // only inputs that break the precondition
        if (lo > hi) lo = hi;
    }
    const uint64_t best = select_split<true>(run, lo, hi, sample_target(b, side, k), own, g.member, group, g.group_base);
    if (own) ws.ywin[g.slot * k + g.member] = best;
}

// the boundary itself, searched inside the brackets
__global__ void __launch_bounds__(256) bracket_partition_kernel(RunTable rt, Workspace ws, uint64_t n_tiles, int group) {
    const GroupLane g = group_lane(group);
    const uint64_t b = g.slot + 1;
    const bool own = b < n_tiles && g.member < (int)rt.k;
    const uint64_t r = b * tile_nominal(rt.k);
    const lsm_entry_t* run = own ? rt.ptr[g.member] : nullptr;
    uint64_t lo = 0, hi = 0, yhi = 0;
    if (own) {
        const uint64_t n = rt.n[g.member];
        const uint64_t ylo = ws.ywin[(2 * (b - 1)) * rt.k + g.member];
        yhi = ws.ywin[(2 * (b - 1) + 1) * rt.k + g.member];
        lo = ylo ? (ylo - 1) * kSampleStride + 1 : 0;
        hi = yhi * kSampleStride;
        if (hi > n) hi = n;
    }
    // no sample above the upper target: the upper bracket proves nothing, search to the end of the runs
    const uint64_t y_total = group_sum_u64(own ? yhi : 0, group);
    if (own && y_total < (r + kSampleStride - 1) / kSampleStride + rt.k) hi = rt.n[g.member];
    if (lo > hi) lo = hi;  // only inputs that break the precondition
    const uint64_t best = select_split<false>(run, lo, hi, r, own, g.member, group, g.group_base);
    if (own) ws.splits[b * rt.k + g.member] = best;
}

// ---------------------------------------------------------------------------------------
// Tile merge.
//
// Every thread owns kMergeItems entries of the tile and keeps their 64 bytes in registers
// from the load to the final store.  What moves through LDS during the merge rounds is one
// 16-byte "surrogate" per entry: the first 14 key bytes (as a 112-bit big-endian number) and
// the entry's tile-local index in the low 16 bits.  Surrogates are merged with stable
// two-way merge-path merges (the left list = lower run indices wins ties).  Afterwards each
// merged position gets the rest of its key (bytes 14..31), its seqno and its type, so that
// neighbours can be compared exactly.  Equal surrogates with different key tails mean the
// 14-byte order was not enough: a short group of such positions is put in key order in place
// (one thread, insertion sort by the tail), and a tile with a longer group is redone by the
// exact path below (ranks by binary search over the tile's pieces with full 32-byte compares).
// ---------------------------------------------------------------------------------------
enum : uint8_t { kFlagEq = 1, kFlagFullEq = 2, kFlagSurvive = 4 };
constexpr int kRepairMax = 32;                // longest prefix-tie group one thread puts in key order
constexpr int kStageEntries = kTileCap / 2;  // output staging: 64 bytes per survivor, two passes at most

struct MergeShared {
    uint4 buf[2][kTileCap];          // surrogate ping-pong; then 2 x uint4 of key tail/seqno/type per position; then output staging
    uint16_t rank[kTileCap];         // tile-local entry index -> merged position
    uint16_t prefix[kTileCap];       // survivors before this merged position
    alignas(4) uint8_t flag[kTileCap + 8];  // per merged position: kFlagEq | kFlagFullEq | kFlagSurvive
    uint32_t seg[LSM_MAX_RUNS + 1];  // start of each run's piece in tile-local index space
    uint64_t lo[LSM_MAX_RUNS];       // first entry of each run's piece
    const lsm_entry_t* run[LSM_MAX_RUNS];  // copy of the run pointers (indexed per lane)
    uint32_t wave_count[kMergeThreads / kWave];
    uint32_t tile;                   // number of the tile inside its compaction (what the look-back counts in)
    uint32_t n;
    uint32_t failed;
    uint32_t inexact;                // some position has an equal surrogate but a different key tail
    uint64_t base;
    // batched compactions only: what the single form takes from its kernel arguments
    uint32_t k, flags, job_tiles, fence_stride;
    lsm_entry_t* out;
    uint64_t* n_out;
    uint64_t* status;
    uint4* fence_out;
};

// The tile kernel has three forms.  Single: one compaction, tile = workgroup, pieces from the split table.
// Range: one tile per key range of a tree - the pieces are the parts of the runs inside the range, found by the
// tile itself, and the survivors go to a fixed slot of the result (no look-back).  Batch: many independent
// compactions in one launch - the workgroup looks up its job, and everything the single form takes from kernel
// arguments comes from the job's descriptor.
enum : int { kModeSingle = 0, kModeRange = 1, kModeBatch = 2 };

struct JobDesc {       // one compaction of a batch (device memory, written by the host)
    uint64_t first_tile;   // number of its first tile in the launch
    uint64_t run_off;      // where its runs start in the run pointer / length arrays
    uint64_t splits_off;   // where its split table starts (in 64-bit words)
    lsm_entry_t* out;
    uint64_t* n_out;
    uint4* fence_out;      // optional fence index of the job's output
    uint32_t n_tiles, k, flags, fence_stride;
};
static_assert(sizeof(JobDesc) == 64, "descriptor layout");

struct ModeArgs {
    // single form: optional filter hashes of the output's keys (kExtras = 2)
    uint64_t* key_hashes;
    // range form
    const uint8_t* lo_keys;   // [n_tiles x 32]
    const uint8_t* hi_keys;
    uint32_t* counts;         // [n_tiles]
    uint32_t max_entries;     // slot pitch of the result
    // batch form
    const uint32_t* tile_job;             // [n_tiles] job of every tile
    const JobDesc* jobs;
    const lsm_entry_t* const* run_ptr;    // runs of all jobs
    const uint64_t* run_n;
};

struct Sur {  // hi = key bytes 0..7, lo = key bytes 8..13 << 16 | index
    uint64_t hi, lo;
};
__device__ __forceinline__ Sur sur_load(const uint4* p) {
    uint4 v = *p;
    Sur r;
    r.hi = ((uint64_t)v.y << 32) | v.x;
    r.lo = ((uint64_t)v.w << 32) | v.z;
    return r;
}
__device__ __forceinline__ void sur_store(uint4* p, const Sur& v) {
    *p = make_uint4((uint32_t)v.hi, (uint32_t)(v.hi >> 32), (uint32_t)v.lo, (uint32_t)(v.lo >> 32));
}
// Where the record of position p sits in the 16-byte-per-position LDS arrays.  Threads own four consecutive
// positions, so lane t of a wave reads or writes position 4t + i: without this every second lane would
// fall on the same banks (64-byte stride).  The swap inside each group of four spreads eight lanes over all banks.
__device__ __forceinline__ uint32_t sw(uint32_t p) { return p ^ ((p >> 3) & 3); }

// a < b as 128-bit numbers (key bits, then index)
__device__ __forceinline__ bool sur_less(const Sur& a, const Sur& b) { return a.hi < b.hi || (a.hi == b.hi && a.lo < b.lo); }
// afterwards a < b
__device__ __forceinline__ void sur_order(Sur& a, Sur& b) {
    const bool swap = sur_less(b, a);
    const Sur t = a;
    a.hi = swap ? b.hi : a.hi;
    a.lo = swap ? b.lo : a.lo;
    b.hi = swap ? t.hi : b.hi;
    b.lo = swap ? t.lo : b.lo;
}
__device__ __forceinline__ bool sur_same_key(const Sur& a, const Sur& b) { return a.hi == b.hi && ((a.lo ^ b.lo) >> 16) == 0; }

// Last j < k with seg[j] <= e (empty pieces share an offset with their successor).  Branch-free;
// top_step = largest power of two below k (0 for k = 1).
__device__ __forceinline__ uint32_t piece_of(const uint32_t* seg, uint32_t k, uint32_t top_step, uint32_t e) {
    uint32_t j = 0;
    for (uint32_t step = top_step; step > 0; step >>= 1) {
        const uint32_t c = j + step;
        const uint32_t v = seg[min(c, k - 1)];
        j = ((c < k) & (v <= e)) ? c : j;
    }
    return j;
}

// Publish this tile's survivor count and return the number of survivors in all earlier tiles
// (decoupled look-back).  Called by wave 0 only, all 64 lanes.  Earlier tiles are earlier
// workgroups, which have started (or finished) by the time this one runs, and will publish; the
// wait is bounded anyway, and a tile that gives up publishes kStFailed, which propagates forward.
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

// order of two entries with the same 14-byte key prefix by the rest of the key, from their info words
__device__ __forceinline__ bool tail_less(const uint4 a0, const uint4 a1, const uint4 b0, const uint4 b1) {
    const uint32_t ta = ((a0.z >> 8) & 0xFF) << 8 | ((a0.z >> 16) & 0xFF), tb = ((b0.z >> 8) & 0xFF) << 8 | ((b0.z >> 16) & 0xFF);
    if (ta != tb) return ta < tb;  // key bytes 14, 15
    const uint64_t a2 = __builtin_bswap64(((uint64_t)a1.y << 32) | a1.x), b2 = __builtin_bswap64(((uint64_t)b1.y << 32) | b1.x);
    if (a2 != b2) return a2 < b2;  // key bytes 16..23
    return __builtin_bswap64(((uint64_t)a1.w << 32) | a1.z) < __builtin_bswap64(((uint64_t)b1.w << 32) | b1.z);
}

// Lower bound of `key` in run[from, n) for a range that is expected to end soon after `from`: doubling steps from
// `from` until a record >= key (or the end) is found, then bisection inside the last step.
__device__ __forceinline__ uint64_t lower_bound_from(const lsm_entry_t* run, uint64_t from, uint64_t n, const Key& key) {
    uint64_t lo = from, step = 16;
    while (lo < n) {
        const uint64_t at = lo + step - 1 < n ? lo + step - 1 : n - 1;  // last record of the step
        if (!key_less(load_key(run + at), key)) {
            bool eq;
            return lower_bound_eq(run, lo, at, key, eq);
        }
        lo = at + 1;
        step <<= 1;
    }
    return n;
}

// two workgroups per compute unit = four waves per SIMD: at most 128 vector registers.
// kExtras: what else the output pass does (compiled out otherwise).  1: rewrites value pointers and / or writes the fence
// index; 2: also writes the filter hash of every survivor's key.
template <int kExtras, int kMode>
__global__ void __launch_bounds__(kMergeThreads) __attribute__((amdgpu_waves_per_eu(4, 4))) merge_kernel(RunTable rt, Workspace ws, uint64_t n_tiles, uint32_t flags_arg,
                                                               lsm_entry_t* out_arg, uint64_t* n_out_arg, const uint64_t* remap_base,
                                                               uint32_t remap_files, uint4* fence_out_arg, uint32_t fence_stride_arg, ModeArgs ma) {
    __shared__ MergeShared s;
    // staging of the survivors' filter hashes (kExtras = 2): the first half lives in s.rank, which is dead by then
    __shared__ uint64_t hash_stage_upper[kExtras == 2 ? kStageEntries / 2 : 1];
    static_assert(sizeof(s.rank) == sizeof(uint64_t) * (kStageEntries / 2), "s.rank holds half a pass of hashes");
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;

    // ---- the tile's k pieces, by wave 0.  Tile number = workgroup number: the look-back below waits only for
    //      tiles with smaller numbers, and workgroups are handed to the compute units in ascending order, so the
    //      tiles waited for are resident or done.  (A ticket taken with an atomic would make that independent
    //      of the dispatch order, but it costs a second dependent memory round trip before the first load: the
    //      tickets come back in a different order than the workgroup numbers for 99 % of the tiles.)  The waits
    //      are bounded in any case.
    if (wave == 0) {
        __builtin_amdgcn_s_setprio(3);  // the other waves wait for this one: let it issue first
        uint64_t t = blockIdx.x;        // tile number inside its compaction
        uint32_t kk = rt.k;
        uint64_t a = 0, b = 0;
        if (kMode == kModeSingle) {
            if (lane < (int)kk) {
                a = ws.splits[t * kk + lane];
                b = ws.splits[(t + 1) * kk + lane];
                s.run[lane] = rt.ptr[lane];
            }
        } else if (kMode == kModeRange) {
            // the part of every run inside [lo_key, hi_key): lane j searches run j
            const Key lo_key = load_key(ma.lo_keys + t * LSM_KEY_BYTES), hi_key = load_key(ma.hi_keys + t * LSM_KEY_BYTES);
            if (lane < (int)kk) {
                const lsm_entry_t* run = rt.ptr[lane];
                const uint64_t len = rt.n[lane];
                bool eq;
                a = len ? lower_bound_eq(run, 0, len, lo_key, eq) : 0;
                b = key_less(lo_key, hi_key) ? lower_bound_from(run, a, len, hi_key) : a;
                s.run[lane] = run;
            }
        } else {
            const JobDesc d = ma.jobs[ma.tile_job[t]];  // the same words for every lane
            kk = d.k;
            t -= d.first_tile;
            if (lane < (int)kk) {
                a = ws.splits[d.splits_off + t * kk + lane];
                b = ws.splits[d.splits_off + (t + 1) * kk + lane];
                s.run[lane] = ma.run_ptr[d.run_off + lane];
            }
            if (lane == 0) {
                s.k = kk;
                s.flags = d.flags;
                s.job_tiles = d.n_tiles;
                s.out = d.out;
                s.n_out = d.n_out;
                s.status = ws.status + d.first_tile;
                s.fence_out = d.fence_out;
                s.fence_stride = d.fence_stride;
            }
        }
        const bool mine = lane < (int)kk;
        // piece lengths -> offsets (inclusive scan over the lanes); split rows never exceed the run
        // lengths, and only inputs that break the precondition can make a row pair inconsistent
        // (a key range may simply hold more than a tile: reported as an overflow of that range)
        const bool bad = mine && (b < a || b - a > (uint64_t)kTileCap);
        uint32_t incl = (mine && !bad) ? (uint32_t)(b - a) : 0;
        for (int off = 1; off < kWave; off <<= 1) {
            const uint32_t v = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += v;
        }
        const uint32_t total = __shfl(incl, kWave - 1, kWave);
        const bool ok = __ballot(bad) == 0 && total <= (uint32_t)kTileCap;
        if (mine) {
            s.lo[lane] = a;
            s.seg[lane + 1] = ok ? incl : 0;
        }
        if (lane == 0) {
            s.seg[0] = 0;
            s.tile = (uint32_t)t;
            s.n = ok ? total : 0;
            s.failed = ok ? 0 : 1;
            s.inexact = 0;
        }
        __builtin_amdgcn_s_setprio(0);
    }
    __syncthreads();
    const uint64_t tile = s.tile;
    if (blockIdx.x >= n_tiles) return;  // cannot happen: the grid has exactly n_tiles workgroups
    const uint32_t n = s.n;
    const uint32_t k = kMode == kModeBatch ? s.k : rt.k;
    const uint32_t flags = kMode == kModeBatch ? s.flags : flags_arg;
    lsm_entry_t* const out = kMode == kModeBatch ? s.out : out_arg;
    uint64_t* const n_out = kMode == kModeBatch ? s.n_out : n_out_arg;
    const uint64_t last_tile = kMode == kModeBatch ? (uint64_t)s.job_tiles - 1 : n_tiles - 1;
    uint4* const fence_out = kMode == kModeBatch ? s.fence_out : fence_out_arg;
    const uint32_t fence_stride = kMode == kModeBatch ? s.fence_stride : fence_stride_arg;
    const uint32_t top_step = k > 1 ? 1u << (31 - __builtin_clz(k - 1)) : 0;

    // ---- load: entry e = tid + i * kMergeThreads stays in this thread's registers until it is stored
    // the few instructions of a memory phase should not queue behind the other workgroup's merge arithmetic
    __builtin_amdgcn_s_setprio(2);
    uint4 ent[kMergeItems][4];
    uint32_t pos[kMergeItems];  // merged position of the entry
    {
        // all addresses first, then all loads, so that the loads of one thread are in flight together
        // (threads without an entry re-read entry 0 and never use it; an unusable tile has n = 0)
        const uint4* src[kMergeItems];
#pragma unroll
        for (int i = 0; i < kMergeItems; i++) {
            const uint32_t e = tid + i * kMergeThreads;
            const uint32_t ee = e < n ? e : 0;
            const uint32_t j = piece_of(s.seg, k, top_step, ee);
            src[i] = reinterpret_cast<const uint4*>(s.run[j] + s.lo[j] + (ee - s.seg[j]));
            pos[i] = 0;
        }
        if (n > 0) {
#pragma unroll
            for (int i = 0; i < kMergeItems; i++)
#pragma unroll
                for (int part = 0; part < 4; part++) ent[i][part] = load_global_u4(src[i] + part);
        } else {
#pragma unroll
            for (int i = 0; i < kMergeItems; i++)
#pragma unroll
                for (int part = 0; part < 4; part++) ent[i][part] = make_uint4(0, 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < kMergeItems; i++) {
        const uint32_t e = tid + i * kMergeThreads;
        if (e < n) {
            Key kk = key_from_raw(ent[i][0], ent[i][1]);
            Sur v;
            v.hi = kk.w[0];
            v.lo = (kk.w[1] & ~0xFFFFull) | e;
            sur_store(&s.buf[0][sw(e)], v);
        }
    }
    if (tid == 0) s.flag[n] = 0;
    __builtin_amdgcn_s_setprio(0);
    __syncthreads();

    // ---- merge rounds: lists of `width` runs each are merged pairwise.  Surrogates are compared as whole
    //      128-bit numbers: the index in the low bits grows with the run number, so the order is the stable one
    //      (equal keys: lower run first) and all values are distinct.  Thread t produces outputs
    //      [4t, 4t + 4): a co-rank search finds where they start in the two lists, then the next four of each
    //      list are read at once and merged in registers (half-cleaner + two exchange stages), so the only
    //      dependent LDS reads of a round are those of the search.
    const uint32_t j_first = piece_of(s.seg, k, top_step, min((uint32_t)(tid * kRoundItems), n ? n - 1 : 0));
    int cur = 0;
    for (uint32_t width = 1; width < k; width <<= 1) {
        const uint4* in = s.buf[cur];
        uint4* dst = s.buf[cur ^ 1];
        uint32_t o = tid * kRoundItems, j = j_first;
        const uint32_t o_end = min(o + (uint32_t)kRoundItems, n);
        while (o < o_end) {
            // the pair of lists whose output range contains position o (o lies in piece j)
            const uint32_t ra = (j / (2 * width)) * 2 * width, rb = min(ra + width, k), rc = min(ra + 2 * width, k);
            const uint32_t sa = s.seg[ra], sb = s.seg[rb], sc = s.seg[rc];
            const uint32_t len_a = sb - sa, len_b = sc - sb;
            const uint32_t stop = min(o_end, sc);
            // co-rank of diagonal d: how many of the first d outputs come from the left list
            const uint32_t d = o - sa;
            uint32_t lo = d > len_b ? d - len_b : 0, hi = min(d, len_a);
            while (lo < hi) {
                const uint32_t mid = (lo + hi) >> 1;
                if (sur_less(sur_load(&in[sw(sa + mid)]), sur_load(&in[sw(sb + (d - 1 - mid))]))) lo = mid + 1;
                else hi = mid;
            }
            const uint32_t a = lo, b = d - lo;
            Sur x[kRoundItems], y[kRoundItems];
#pragma unroll
            for (int i = 0; i < kRoundItems; i++) {
                x[i] = sur_load(&in[sw(min(sa + a + i, (uint32_t)kTileCap - 1))]);
                y[i] = sur_load(&in[sw(min(sb + b + i, (uint32_t)kTileCap - 1))]);
                if (a + i >= len_a) x[i].hi = x[i].lo = ~0ull;  // past the end of a list: larger than any surrogate
                if (b + i >= len_b) y[i].hi = y[i].lo = ~0ull;
            }
            // the four smallest of x[0..3], y[0..3] in order
            Sur c[kRoundItems];
#pragma unroll
            for (int i = 0; i < kRoundItems; i++) c[i] = sur_less(x[i], y[kRoundItems - 1 - i]) ? x[i] : y[kRoundItems - 1 - i];
            sur_order(c[0], c[2]);
            sur_order(c[1], c[3]);
            sur_order(c[0], c[1]);
            sur_order(c[2], c[3]);
#pragma unroll
            for (int i = 0; i < kRoundItems; i++)
                if (o + i < stop) sur_store(&dst[sw(o + i)], c[i]);
            o = stop;
            for (j = rc; j + 1 < k && s.seg[j + 1] <= o; j++) {}  // piece of the next position (skips empty pieces)
        }
        __syncthreads();
        cur ^= 1;
    }

    // ---- merged position p <-> entry index; does p repeat the 14-byte key prefix of p-1?
    {
        const uint4* fin = s.buf[cur];
        const uint32_t o0 = tid * kMergeItems;
        if (o0 < n) {
            Sur prev = sur_load(&fin[sw(o0 > 0 ? o0 - 1 : 0)]);
            for (uint32_t o = o0; o < min(o0 + (uint32_t)kMergeItems, n); o++) {
                Sur v = sur_load(&fin[sw(o)]);
                s.flag[o] = (o > 0 && sur_same_key(prev, v)) ? kFlagEq : 0;
                s.rank[v.lo & 0xFFFF] = (uint16_t)o;
                prev = v;
            }
        }
    }
    __syncthreads();

    // ---- every owner posts key bytes 14..31, seqno and type of its entries at their merged positions
    uint4* info0 = s.buf[0];  // {seqno lo, seqno hi, type | key bytes 14..15 << 8, entry index} of the entry at a position
    uint4* info1 = s.buf[1];  // its key bytes 16..31
#pragma unroll
    for (int i = 0; i < kMergeItems; i++) {
        const uint32_t e = tid + i * kMergeThreads;
        if (e < n) {
            const uint32_t p = s.rank[e];
            pos[i] = p;
            info0[sw(p)] = make_uint4(ent[i][2].x, ent[i][2].y, (ent[i][2].z & 0xFF) | (ent[i][0].w & 0xFFFF0000u) >> 8, e);
            info1[sw(p)] = ent[i][1];
        }
    }
    __syncthreads();

    // ---- exact equality with the previous position; a differing tail under an equal prefix makes the tile inexact.
    //      A thread's four positions are neighbours, so the words of positions o0-1 .. o0+3 that some comparison
    //      needs are all requested before the first compare.
    {
        const uint32_t o0 = tid * kMergeItems;
        if (o0 < n) {
            const uint32_t f = *reinterpret_cast<const uint32_t*>(&s.flag[o0]);
            bool eq[kMergeItems + 1];
#pragma unroll
            for (int i = 0; i < kMergeItems; i++) eq[i] = o0 + i < n && ((f >> (8 * i)) & kFlagEq) != 0;
            eq[kMergeItems] = false;
            uint32_t z[kMergeItems + 1];
            uint4 t[kMergeItems + 1];  // [i] = position o0 + i - 1
#pragma unroll
            for (int i = 0; i <= kMergeItems; i++) {
                const bool need = (i > 0 && eq[i - 1]) || eq[i];  // compared as a position or as a predecessor
                z[i] = 0;
                t[i] = make_uint4(0, 0, 0, 0);
                if (need) {
                    z[i] = info0[sw(o0 + i - 1)].z;
                    t[i] = info1[sw(o0 + i - 1)];
                }
            }
            uint32_t g = f;
            bool inexact = false;
#pragma unroll
            for (int i = 0; i < kMergeItems; i++) {
                if (eq[i]) {
                    const bool same = ((z[i + 1] ^ z[i]) >> 8) == 0 && t[i + 1].x == t[i].x && t[i + 1].y == t[i].y &&
                                      t[i + 1].z == t[i].z && t[i + 1].w == t[i].w;
                    g |= same ? (uint32_t)kFlagFullEq << (8 * i) : 0;
                    inexact = inexact || !same;
                }
            }
            if (g != f) *reinterpret_cast<uint32_t*>(&s.flag[o0]) = g;
            if (inexact) s.inexact = 1;
        }
    }
    __syncthreads();

    if (s.inexact != 0) {
        // ---- repair: positions that share the 14-byte prefix but not the whole key stand in run order, not in
        //      key order.  The thread whose share holds the first position of such a group sorts the group by the
        //      rest of the key (stable, so equal keys keep their run order); a group too long for one thread
        //      sends the whole tile to the exact path instead.
        const uint32_t o0 = tid * kMergeItems;
        for (uint32_t o = o0; o < min(o0 + (uint32_t)kMergeItems, n); o++) {
            if ((s.flag[o] & kFlagEq) != 0 || (s.flag[o + 1] & kFlagEq) == 0) continue;  // flag[n] is 0
            uint32_t end = o + 1;
            bool broken = false;
            for (; s.flag[end] & kFlagEq; end++) broken = broken || (s.flag[end] & kFlagFullEq) == 0;
            if (!broken) continue;
            if (end - o > (uint32_t)kRepairMax) {
                s.inexact = 2;
                continue;
            }
            for (uint32_t a = o + 1; a < end; a++) {
                const uint4 x0 = info0[sw(a)], x1 = info1[sw(a)];
                uint32_t b = a;
                for (; b > o && tail_less(x0, x1, info0[sw(b - 1)], info1[sw(b - 1)]); b--) {
                    info0[sw(b)] = info0[sw(b - 1)];
                    info1[sw(b)] = info1[sw(b - 1)];
                }
                info0[sw(b)] = x0;
                info1[sw(b)] = x1;
            }
            s.rank[info0[sw(o)].w] = (uint16_t)o;
            for (uint32_t a = o + 1; a < end; a++) {
                const bool same = !tail_less(info0[sw(a - 1)], info1[sw(a - 1)], info0[sw(a)], info1[sw(a)]);  // sorted: not less = equal
                s.flag[a] = same ? (kFlagEq | kFlagFullEq) : kFlagEq;
                s.rank[info0[sw(a)].w] = (uint16_t)a;
            }
        }
        __syncthreads();
        if (s.inexact == 1) {
#pragma unroll
            for (int i = 0; i < kMergeItems; i++) {
                const uint32_t e = tid + i * kMergeThreads;
                if (e < n) pos[i] = s.rank[e];
            }
        }
    }

    if (s.inexact != 2) {
        // ---- survivors: newest version of each key (largest seqno, ties to the earlier = lower run),
        //      minus winning tombstones when the output is the last level.  Groups of equal keys are short and
        //      mostly lie inside a thread's four positions: those are settled from registers, and only a
        //      group that crosses into a neighbour's share is followed through LDS.
        const uint32_t o0 = tid * kMergeItems;
        if (o0 < n) {
            const uint32_t f = *reinterpret_cast<const uint32_t*>(&s.flag[o0]);
            const bool more = o0 + kMergeItems < n && (s.flag[o0 + kMergeItems] & kFlagFullEq) != 0;  // the group goes on to the right
            bool fe[kMergeItems];
            uint64_t seq[kMergeItems];
            uint32_t type[kMergeItems];
#pragma unroll
            for (int i = 0; i < kMergeItems; i++) {
                const bool valid = o0 + i < n;
                const uint4 me = info0[sw(valid ? o0 + i : o0)];
                fe[i] = valid && ((f >> (8 * i)) & kFlagFullEq) != 0;
                seq[i] = ((uint64_t)me.y << 32) | me.x;
                type[i] = me.z & 0xFF;
            }
            uint32_t g = f;
#pragma unroll
            for (int i = 0; i < kMergeItems; i++) {
                bool win = true, chain = true;
#pragma unroll
                for (int q = i; q >= 1; q--) {  // earlier members of the group
                    chain = chain && fe[q];
                    if (chain && seq[q - 1] >= seq[i]) win = false;
                }
                if (chain && fe[0])
                    for (uint32_t p = o0; s.flag[p] & kFlagFullEq; p--) {  // flag[0] never has the bit
                        const uint4 v = info0[sw(p - 1)];
                        if ((((uint64_t)v.y << 32) | v.x) >= seq[i]) win = false;
                    }
                chain = true;
#pragma unroll
                for (int q = i + 1; q < kMergeItems; q++) {  // later members
                    chain = chain && fe[q];
                    if (chain && seq[q] > seq[i]) win = false;
                }
                if (chain && more)
                    for (uint32_t p = o0 + kMergeItems; s.flag[p] & kFlagFullEq; p++) {  // flag[n] is 0
                        const uint4 v = info0[sw(p)];
                        if ((((uint64_t)v.y << 32) | v.x) > seq[i]) win = false;
                    }
                if (win && (flags & LSM_BOTTOMMOST) && type[i] == LSM_TOMBSTONE) win = false;
                if (win && o0 + i < n) g |= (uint32_t)kFlagSurvive << (8 * i);
            }
            if (g != f) *reinterpret_cast<uint32_t*>(&s.flag[o0]) = g;
        }
    } else {
        // ---- exact path: merged position and winner of every entry by binary search over the
        //      tile's other pieces with full 32-byte compares, order (key, run index).  The keys
        //      are staged in LDS in entry order (the info arrays are not needed any more), so only
        //      the seqno of an equal key in another piece is read from global memory.
        __syncthreads();
        uint4* klo = s.buf[0];  // key bytes 0..15 of entry e
        uint4* khi = s.buf[1];  // key bytes 16..31
#pragma unroll
        for (int i = 0; i < kMergeItems; i++) {
            const uint32_t e = tid + i * kMergeThreads;
            if (e < n) {
                klo[e] = ent[i][0];
                khi[e] = ent[i][1];
            }
        }
        for (uint32_t o = tid; o <= n; o += kMergeThreads) s.flag[o] = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kMergeItems; i++) {
            const uint32_t e = tid + i * kMergeThreads;
            if (e < n) {
                const uint32_t j = piece_of(s.seg, k, top_step, e);
                const Key x = key_from_raw(ent[i][0], ent[i][1]);
                const uint64_t seq = ((uint64_t)ent[i][2].y << 32) | ent[i][2].x;
                uint32_t p = e - s.seg[j];
                bool win = true;
                for (uint32_t j2 = 0; j2 < k; j2++) {
                    if (j2 == j) continue;
                    const uint32_t first = s.seg[j2], last = s.seg[j2 + 1];
                    uint32_t lb = first, ub = last;
                    while (lb < ub) {
                        const uint32_t mid = (lb + ub) >> 1;
                        if (entry_key_less(&klo[mid], &khi[mid], x)) lb = mid + 1;
                        else ub = mid;
                    }
                    p += lb - first;
                    if (lb < last && key_equal(key_from_raw(klo[lb], khi[lb]), x)) {
                        const uint64_t other = s.run[j2][s.lo[j2] + (lb - first)].seqno;
                        if (other > seq || (other == seq && j2 < j)) win = false;
                        if (j2 < j) p++;
                    }
                }
                if (win && (flags & LSM_BOTTOMMOST) && (ent[i][2].z & 0xFF) == LSM_TOMBSTONE) win = false;
                pos[i] = p;
                if (win) s.flag[p] = kFlagSurvive;
            }
        }
    }
    __syncthreads();

    // ---- survivors before each merged position (block-wide exclusive prefix sum in position order)
    uint32_t total = 0;
    {
        const uint32_t o0 = tid * kMergeItems;
        uint32_t my_count = 0;
        for (uint32_t o = o0; o < min(o0 + (uint32_t)kMergeItems, n); o++) my_count += (s.flag[o] & kFlagSurvive) ? 1 : 0;
        uint32_t incl = my_count;
        for (int off = 1; off < kWave; off <<= 1) {
            uint32_t v = __shfl_up(incl, off, kWave);
            if (lane >= off) incl += v;
        }
        if (lane == kWave - 1) s.wave_count[wave] = incl;
        __syncthreads();
        uint32_t before = incl - my_count;
        for (int w = 0; w < kMergeThreads / kWave; w++) {
            const uint32_t c = s.wave_count[w];
            if (w < wave) before += c;
            total += c;
        }
        for (uint32_t o = o0; o < min(o0 + (uint32_t)kMergeItems, n); o++) {
            s.prefix[o] = (uint16_t)before;
            before += (s.flag[o] & kFlagSurvive) ? 1 : 0;
        }
    }

    __syncthreads();  // prefix[] complete, last reads of info[] done: the staging area is free

    // ---- output offset of this tile: wave 0 looks back while the other waves already stage their survivors
    if (wave == 0) {
        __builtin_amdgcn_s_setprio(3);  // the stores of the whole tile wait for this wave
        bool failed;
        uint64_t base;
        if (kMode == kModeRange) {
            // a range has its own slot of max_entries entries; one that holds more (or more than a tile) is reported
            base = tile * (uint64_t)ma.max_entries;
            failed = s.failed != 0 || total > ma.max_entries;
            if (lane == 0) ma.counts[tile] = failed ? ~0u : total;
        } else {
            base = lookback(kMode == kModeBatch ? s.status : ws.status, tile, total, s.failed != 0, &failed);
        }
        if (lane == 0) {
            s.base = base;
            if (failed) s.failed = 1;
        }
    }

    // ---- survivors leave through an LDS stage so that the global stores are contiguous; the four
    //      16-byte parts of a slot are rotated by the slot number to spread them over the banks
    uint4* stage = &s.buf[0][0];
    __builtin_amdgcn_s_setprio(2);  // output is a memory phase again
    uint64_t base = 0;
    uint32_t first = 0;
    do {
#pragma unroll
        for (int i = 0; i < kMergeItems; i++) {
            const uint32_t e = tid + i * kMergeThreads;
            if (e < n && (s.flag[pos[i]] & kFlagSurvive)) {
                // pointer rewrite for merged tensor files (paper section 3.4): vptr = base[file] + offset
                if (kExtras && first == 0 && remap_files != 0 && (ent[i][2].z & 0xFF) == LSM_PUT && ent[i][3].y < remap_files) {
                    const uint64_t v = remap_base[ent[i][3].y] + ent[i][3].x;
                    ent[i][3].x = (uint32_t)v;
                    ent[i][3].y = (uint32_t)(v >> 32);
                }
                const uint32_t slot = (uint32_t)s.prefix[pos[i]] - first;  // wraps for slots before this pass
                if (slot < (uint32_t)kStageEntries) {
#pragma unroll
                    for (int part = 0; part < 4; part++) stage[slot * 4 + (part ^ (slot & 3))] = ent[i][part];
                    // the filter hash of the survivor's key travels with it (paper section 2.2: a new run gets its Bloom
                    // filter; the filter is then built from these 8-byte values, not from the run)
                    if (kExtras == 2 && kMode == kModeSingle && ma.key_hashes != nullptr) {
                        const uint64_t h = bloom_key_hash(key_from_raw(ent[i][0], ent[i][1]));
                        if (slot < (uint32_t)kStageEntries / 2) reinterpret_cast<uint64_t*>(s.rank)[slot] = h;
                        else hash_stage_upper[slot - kStageEntries / 2] = h;
                    }
                }
            }
        }
        __syncthreads();
        if (first == 0) {
            const bool failed = s.failed != 0;
            base = s.base;
            if (kMode != kModeRange && tile == last_tile && tid == 0) *n_out = failed ? ~0ull : base + total;
            if (failed) return;
        }
        const uint32_t count = min(total - first, (uint32_t)kStageEntries);
        uint4* dst = reinterpret_cast<uint4*>(out + base + first);
        for (uint32_t c = tid; c < count * 4; c += kMergeThreads) {
            const uint32_t part = (c ^ (c >> 2)) & 3;  // which 16 bytes of the entry stage[c] holds
            const uint4 v = stage[c];
            dst[(c & ~3u) | part] = v;
            // fence index of the new run: the key of every fence_stride-th output entry
            if (kExtras && fence_out != nullptr && part < 2) {
                const uint64_t at = base + first + (c >> 2);
                if (at % fence_stride == 0) fence_out[(at / fence_stride) * 2 + part] = v;
            }
        }
        if (kExtras == 2 && kMode == kModeSingle && ma.key_hashes != nullptr) {
            for (uint32_t c = tid; c < count; c += kMergeThreads)
                ma.key_hashes[base + first + c] = c < (uint32_t)kStageEntries / 2 ? reinterpret_cast<const uint64_t*>(s.rank)[c]
                                                                                  : hash_stage_upper[c - kStageEntries / 2];
        }
        first += kStageEntries;
        if (first < total) __syncthreads();  // the stage is reused
    } while (first < total);
}

// ---------------------------------------------------------------------------------------
// Partition of a batch of independent compactions: one group of lanes per tile of the launch.  The group of a
// job's tile number t > 0 searches boundary t over the job's whole runs (the jobs of a batch are small); the groups
// of a job's first and last tile also write the first (all zero) and the last (run lengths) row of its split table,
// and every group clears its tile's status word.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) partition_batch_kernel(Workspace ws, ModeArgs ma, uint64_t n_tiles, int group) {
    const GroupLane g = group_lane(group);
    const bool live = g.slot < n_tiles;
    JobDesc d = {};
    if (live) d = ma.jobs[ma.tile_job[g.slot]];
    const uint64_t t = live ? g.slot - d.first_tile : 0;
    const bool own = live && g.member < (int)d.k;
    const lsm_entry_t* run = own ? ma.run_ptr[d.run_off + g.member] : nullptr;
    const uint64_t len = own ? ma.run_n[d.run_off + g.member] : 0;
    const bool search = t > 0;  // the same for all lanes of a group
    uint64_t best = 0;
    if (d.k == 2) {  // the two lanes of the group walk the merge path together (the same reads) and keep one bound each
        if (own && search) {
            uint64_t ia, ib;
            split_two(ma.run_ptr[d.run_off], ma.run_n[d.run_off], ma.run_ptr[d.run_off + 1], ma.run_n[d.run_off + 1], t * tile_nominal(2), ia, ib);
            best = g.member == 0 ? ia : ib;
        }
    } else {
        best = select_split<false>(run, 0, (own && search) ? len : 0, t * tile_nominal(d.k ? d.k : 1), own && search, g.member, group, g.group_base);
    }
    if (own) {
        uint64_t* rows = ws.splits + d.splits_off;
        rows[t * d.k + g.member] = search ? best : 0;
        if (t + 1 == d.n_tiles) rows[(t + 1) * d.k + g.member] = len;
    }
    if (live && g.member == 0) ws.status[g.slot] = 0;
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

static uint64_t tiles_for(uint64_t total, uint32_t k) { return (total + tile_nominal(k) - 1) / tile_nominal(k); }
static uint64_t coarse_rows(uint64_t n_tiles) { return n_tiles > 1 ? (n_tiles - 1) / kCoarseStride : 0; }

// Lays the workspace out; with base == nullptr it only measures.  Returns the bytes used.
static size_t carve(void* base, const uint64_t* run_lens, uint32_t k, Workspace* ws) {
    uint64_t total = 0;
    for (uint32_t j = 0; j < k; j++) total += run_lens[j];
    const uint64_t n_tiles = tiles_for(total, k), n_coarse = coarse_rows(n_tiles);
    char* p = static_cast<char*>(base);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* at = p ? p + off : nullptr;
        off += align256(bytes);
        return at;
    };
    Workspace w;
    w.hdr = reinterpret_cast<Header*>(take(sizeof(Header)));
    w.status = reinterpret_cast<uint64_t*>(take(n_tiles * sizeof(uint64_t)));
    w.splits = reinterpret_cast<uint64_t*>(take((n_tiles + 1) * (uint64_t)k * sizeof(uint64_t)));
    w.ycoarse = reinterpret_cast<uint64_t*>(take((n_coarse + 2) * (uint64_t)k * sizeof(uint64_t)));
    w.ywin = reinterpret_cast<uint64_t*>(take(2 * (n_tiles ? n_tiles - 1 : 0) * (uint64_t)k * sizeof(uint64_t)));
    for (uint32_t j = 0; j < LSM_MAX_RUNS; j++) {
        w.st.m[j] = j < k ? (run_lens[j] + kSampleStride - 1) / kSampleStride : 0;
        w.st.ptr[j] = j < k ? reinterpret_cast<SampleKey*>(take(w.st.m[j] * sizeof(SampleKey))) : nullptr;
    }
    if (ws) *ws = w;
    return off;
}

}  // namespace lsm

extern "C" size_t lsm_compact_workspace_bytes(const uint64_t* run_lens, uint32_t n_runs) {
    if (run_lens == nullptr || n_runs == 0 || n_runs > LSM_MAX_RUNS) return 0;
    return lsm::carve(nullptr, run_lens, n_runs, nullptr);
}

extern "C" int lsm_compact(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                           size_t workspace_bytes, void* stream) {
    return lsm_compact_timed(runs, n_runs, flags, out, workspace, workspace_bytes, stream, nullptr);
}

extern "C" int lsm_compact_timed(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                                 size_t workspace_bytes, void* stream_v, const lsm_compact_events_t* ev) {
    return lsm_compact_remap(runs, n_runs, flags, out, workspace, workspace_bytes, stream_v, nullptr, ev);
}

namespace lsm {

// Enqueues the kernels of one compaction.  rt.n are the run lengths the launch sizes are taken from.
static int launch_compaction(const RunTable& rt, uint32_t flags, const lsm_out_t* out, void* workspace, hipStream_t stream,
                             const uint64_t* remap_base, uint32_t remap_files, const lsm_compact_events_t* ev) {
    const uint32_t n_runs = rt.k;
    uint64_t total = 0;
    for (uint32_t j = 0; j < n_runs; j++) total += rt.n[j];
    const uint64_t n_tiles = tiles_for(total, n_runs);
    if (n_tiles >= (1ull << 31)) return LSM_ERR_BAD_ARG;
    Workspace ws;
    carve(workspace, rt.n, n_runs, &ws);
    const uint64_t n_coarse = coarse_rows(n_tiles);  // boundaries kCoarseStride, 2 * kCoarseStride, ... < n_tiles

    // a compaction of a few tiles that is not validated: the partition launch does the clearing as well
    const bool direct = n_tiles > 1 && (n_tiles < kSampledMinTiles || n_runs == 2);  // two runs: bisection on the merge path at any size
    const bool fused_init = direct && !(flags & LSM_VALIDATE);
    if (!fused_init) {
        uint32_t init_blocks = (uint32_t)((n_tiles + 255) / 256);
        if (init_blocks == 0) init_blocks = 1;
        if (init_blocks > 1024) init_blocks = 1024;
        hipLaunchKernelGGL(init_kernel, dim3(init_blocks), dim3(256), 0, stream, rt, ws, n_tiles, n_coarse, out->n_out);
    }

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
        int group = 1;
        while (group < (int)n_runs) group <<= 1;
        const uint64_t per_block = (uint64_t)(256 / kWave) * (kWave / group);  // selection problems per workgroup
        auto blocks = [&](uint64_t problems) { return dim3((uint32_t)((problems + per_block - 1) / per_block)); };
        if (direct) {
            // a few dozen boundaries: every one searched over whole runs (a coarse pass first would be a second
            // dependent launch, which costs more than the longer searches)
            const bool brief = total <= kShortRunsTotal;
            if (fused_init && brief) hipLaunchKernelGGL((partition_kernel<true, true>), blocks(n_tiles - 1), dim3(256), 0, stream, rt, ws, n_tiles, group);
            else if (fused_init) hipLaunchKernelGGL((partition_kernel<true, false>), blocks(n_tiles - 1), dim3(256), 0, stream, rt, ws, n_tiles, group);
            else if (brief) hipLaunchKernelGGL((partition_kernel<false, true>), blocks(n_tiles - 1), dim3(256), 0, stream, rt, ws, n_tiles, group);
            else hipLaunchKernelGGL((partition_kernel<false, false>), blocks(n_tiles - 1), dim3(256), 0, stream, rt, ws, n_tiles, group);
        } else {
            uint64_t m_max = 0;
            for (uint32_t j = 0; j < n_runs; j++) m_max = ws.st.m[j] > m_max ? ws.st.m[j] : m_max;
            uint64_t sample_blocks = (2 * m_max + 255) / 256;
            if (sample_blocks > 4096) sample_blocks = 4096;
            hipLaunchKernelGGL(sample_kernel, dim3((uint32_t)sample_blocks, n_runs), dim3(256), 0, stream, rt, ws.st);
            hipLaunchKernelGGL(sample_coarse_kernel, blocks(n_coarse), dim3(256), 0, stream, ws, n_runs, n_coarse, group);
            hipLaunchKernelGGL(sample_fine_kernel, blocks(2 * (n_tiles - 1)), dim3(256), 0, stream, ws, n_runs, n_tiles, n_coarse, group);
            hipLaunchKernelGGL(bracket_partition_kernel, blocks(n_tiles - 1), dim3(256), 0, stream, rt, ws, n_tiles, group);
        }
    }
    if (ev && ev->before_merge && hipEventRecord(static_cast<hipEvent_t>(ev->before_merge), stream) != hipSuccess)
        return LSM_ERR_HIP;
    if (n_tiles > 0) {
        uint4* const fence_out = reinterpret_cast<uint4*>(out->fence_keys);
        const uint32_t fence_stride = out->fence_keys ? out->fence_stride : 1u;
        ModeArgs extras = {};
        extras.key_hashes = out->key_hashes;
        if (out->key_hashes != nullptr)
            hipLaunchKernelGGL((merge_kernel<2, kModeSingle>), dim3((uint32_t)n_tiles), dim3(kMergeThreads), 0, stream, rt, ws, n_tiles, flags,
                               out->entries, out->n_out, remap_base, remap_files, fence_out, fence_stride, extras);
        else if (remap_files != 0 || fence_out != nullptr)
            hipLaunchKernelGGL((merge_kernel<1, kModeSingle>), dim3((uint32_t)n_tiles), dim3(kMergeThreads), 0, stream, rt, ws, n_tiles, flags,
                               out->entries, out->n_out, remap_base, remap_files, fence_out, fence_stride, ModeArgs{});
        else
            hipLaunchKernelGGL((merge_kernel<0, kModeSingle>), dim3((uint32_t)n_tiles), dim3(kMergeThreads), 0, stream, rt, ws, n_tiles, flags,
                               out->entries, out->n_out, remap_base, remap_files, fence_out, fence_stride, ModeArgs{});
    }
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

int compact_device_lengths(const lsm_entry_t* const* ptr, const uint64_t* n_upper, const uint64_t* n_dev, uint32_t k, uint32_t flags,
                           const lsm_out_t* out, void* workspace, size_t workspace_bytes, hipStream_t stream) {
    if (k == 0 || k > LSM_MAX_RUNS || (flags & LSM_VALIDATE)) return LSM_ERR_BAD_ARG;
    if (workspace == nullptr || workspace_bytes < lsm_compact_workspace_bytes(n_upper, k)) return LSM_ERR_WORKSPACE;
    RunTable rt;
    rt.k = k;
    rt.n_dev = n_dev;
    uint64_t total = 0;
    for (uint32_t j = 0; j < LSM_MAX_RUNS; j++) {
        rt.ptr[j] = j < k ? ptr[j] : nullptr;
        rt.n[j] = j < k ? n_upper[j] : 0;
        total += rt.n[j];
    }
    // with lengths that are only bounds the sampled partition would copy samples from beyond the runs' ends
    if (tiles_for(total, k) >= kSampledMinTiles) return LSM_ERR_BAD_ARG;
    return launch_compaction(rt, flags, out, workspace, stream, nullptr, 0, nullptr);
}

}  // namespace lsm

extern "C" int lsm_compact_remap(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                                 size_t workspace_bytes, void* stream_v, const lsm_remap_t* remap, const lsm_compact_events_t* ev) {
    using namespace lsm;
    if (remap != nullptr && remap->n_files != 0 && remap->base == nullptr) return LSM_ERR_NULL;
    const uint64_t* remap_base = remap ? remap->base : nullptr;
    const uint32_t remap_files = remap ? remap->n_files : 0;
    if (runs == nullptr || out == nullptr || out->n_out == nullptr) return LSM_ERR_NULL;
    if (n_runs == 0 || n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    RunTable rt;
    rt.k = n_runs;
    rt.n_dev = nullptr;
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
    if (out->fence_keys != nullptr && (out->fence_stride == 0 || (reinterpret_cast<uintptr_t>(out->fence_keys) & 15) != 0))
        return LSM_ERR_BAD_ARG;
    if ((reinterpret_cast<uintptr_t>(out->key_hashes) & 7) != 0) return LSM_ERR_BAD_ARG;
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 ||
        workspace_bytes < lsm_compact_workspace_bytes(rt.n, n_runs))
        return LSM_ERR_WORKSPACE;
    return launch_compaction(rt, flags, out, workspace, static_cast<hipStream_t>(stream_v), remap_base, remap_files, ev);
}

// ---------------------------------------------------------------------------------------
// lsm_range_scan: the live content of many key ranges of a tree, one tile per range.
// ---------------------------------------------------------------------------------------
extern "C" int lsm_range_scan(const lsm_ranges_t* ranges, const lsm_tree_t* tree, const lsm_range_out_t* out, void* stream_v) {
    using namespace lsm;
    if (ranges == nullptr || tree == nullptr || out == nullptr) return LSM_ERR_NULL;
    if (ranges->max_entries == 0 || ranges->max_entries > LSM_RANGE_MAX_ENTRIES || tree->n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    if (ranges->n_ranges == 0) return LSM_OK;
    if (ranges->lo_keys == nullptr || ranges->hi_keys == nullptr || out->entries == nullptr || out->counts == nullptr) return LSM_ERR_NULL;
    if (((reinterpret_cast<uintptr_t>(ranges->lo_keys) | reinterpret_cast<uintptr_t>(ranges->hi_keys)) & 15) != 0 ||
        (reinterpret_cast<uintptr_t>(out->entries) & 63) != 0)
        return LSM_ERR_BAD_ARG;
    if (tree->n_runs > 0 && tree->runs == nullptr) return LSM_ERR_NULL;
    RunTable rt;
    rt.k = tree->n_runs ? tree->n_runs : 1;  // a tree without runs: one empty run
    rt.n_dev = nullptr;
    for (uint32_t j = 0; j < LSM_MAX_RUNS; j++) {
        rt.ptr[j] = nullptr;
        rt.n[j] = 0;
    }
    for (uint32_t j = 0; j < tree->n_runs; j++) {
        const lsm_run_t& r = tree->runs[j].run;
        if (r.n > 0 && r.entries == nullptr) return LSM_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(r.entries) & 63) != 0) return LSM_ERR_BAD_ARG;
        rt.ptr[j] = r.entries;
        rt.n[j] = r.n;
    }
    ModeArgs ma = {};
    ma.lo_keys = ranges->lo_keys;
    ma.hi_keys = ranges->hi_keys;
    ma.counts = out->counts;
    ma.max_entries = ranges->max_entries;
    Workspace ws = {};
    hipLaunchKernelGGL((merge_kernel<0, kModeRange>), dim3(ranges->n_ranges), dim3(kMergeThreads), 0, static_cast<hipStream_t>(stream_v), rt, ws,
                       (uint64_t)ranges->n_ranges, (uint32_t)LSM_BOTTOMMOST, out->entries, (uint64_t*)nullptr, (const uint64_t*)nullptr, 0u,
                       (uint4*)nullptr, 1u, ma);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

// ---------------------------------------------------------------------------------------
// lsm_compact_batch: many independent small compactions in two launches.
// Workspace: tile status words | split tables of all jobs | the table the host builds (job of every tile, job
// descriptors, run pointers, run lengths).
// ---------------------------------------------------------------------------------------
namespace lsm {
struct BatchLayout {
    uint64_t tiles, split_words, runs;
    size_t status, splits, tile_job, jobs, run_ptr, run_n, total;
    uint32_t k_max;
};
// Pinned host memory for the job table of one thread, with an event that tells when the last copy out of it is done.
struct BatchStaging {
    unsigned char* mem = nullptr;
    size_t capacity = 0;
    hipEvent_t copied = nullptr;
    bool pending = false;

    unsigned char* acquire(size_t bytes) {
        if (pending && hipEventSynchronize(copied) != hipSuccess) return nullptr;
        pending = false;
        if (copied == nullptr && hipEventCreateWithFlags(&copied, hipEventDisableTiming) != hipSuccess) return nullptr;
        if (bytes > capacity) {
            if (mem != nullptr) (void)hipHostFree(mem);
            mem = nullptr;
            capacity = 0;
            const size_t want = bytes < (1u << 16) ? (1u << 16) : bytes + bytes / 2;
            void* p = nullptr;
            if (hipHostMalloc(&p, want, hipHostMallocDefault) != hipSuccess) return nullptr;
            mem = static_cast<unsigned char*>(p);
            capacity = want;
        }
        return mem;
    }
    bool copy_enqueued(hipStream_t stream) {
        if (hipEventRecord(copied, stream) != hipSuccess) return false;
        pending = true;
        return true;
    }
    // no destructor: at thread or process exit the HIP runtime may already be gone; the memory goes with the process
};

static int batch_layout(const lsm_compact_job_t* jobs, uint32_t n_jobs, BatchLayout* l) {
    l->tiles = l->split_words = l->runs = 0;
    l->k_max = 1;
    for (uint32_t j = 0; j < n_jobs; j++) {
        const lsm_compact_job_t& job = jobs[j];
        if (job.runs == nullptr) return LSM_ERR_NULL;
        if (job.n_runs == 0 || job.n_runs > LSM_MAX_RUNS || (job.flags & LSM_VALIDATE)) return LSM_ERR_BAD_ARG;
        if (job.out.fence_keys != nullptr && (job.out.fence_stride == 0 || (reinterpret_cast<uintptr_t>(job.out.fence_keys) & 15) != 0))
            return LSM_ERR_BAD_ARG;
        if (job.out.key_hashes != nullptr) return LSM_ERR_BAD_ARG;  // filters of a batch: lsm_build_bloom_batch
        uint64_t total = 0;
        for (uint32_t r = 0; r < job.n_runs; r++) total += job.runs[r].n;
        uint64_t nt = tiles_for(total, job.n_runs);
        if (nt >= kSampledMinTiles) return LSM_ERR_BAD_ARG;  // a large compaction: lsm_compact
        if (nt == 0) nt = 1;                                  // an empty job keeps one (empty) tile, which writes its count
        l->tiles += nt;
        l->split_words += (nt + 1) * job.n_runs;
        l->runs += job.n_runs;
        if (job.n_runs > l->k_max) l->k_max = job.n_runs;
    }
    if (l->tiles >= (1ull << 31)) return LSM_ERR_BAD_ARG;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align256(bytes);
        return at;
    };
    l->status = take(l->tiles * sizeof(uint64_t));
    l->splits = take(l->split_words * sizeof(uint64_t));
    l->tile_job = take(l->tiles * sizeof(uint32_t));  // from here on: written by the host, one copy
    l->jobs = take((size_t)n_jobs * sizeof(JobDesc));
    l->run_ptr = take(l->runs * sizeof(void*));
    l->run_n = take(l->runs * sizeof(uint64_t));
    l->total = off;
    return LSM_OK;
}
}  // namespace lsm

extern "C" size_t lsm_compact_batch_workspace_bytes(const lsm_compact_job_t* jobs, uint32_t n_jobs) {
    lsm::BatchLayout l;
    if (jobs == nullptr || n_jobs == 0 || lsm::batch_layout(jobs, n_jobs, &l) != LSM_OK) return 0;
    return l.total;
}

extern "C" int lsm_compact_batch(const lsm_compact_job_t* jobs, uint32_t n_jobs, void* workspace, size_t workspace_bytes, void* stream_v) {
    using namespace lsm;
    if (n_jobs == 0) return LSM_OK;
    if (jobs == nullptr) return LSM_ERR_NULL;
    BatchLayout l;
    const int rc = batch_layout(jobs, n_jobs, &l);
    if (rc != LSM_OK) return rc;
    for (uint32_t j = 0; j < n_jobs; j++) {
        const lsm_compact_job_t& job = jobs[j];
        uint64_t total = 0;
        for (uint32_t r = 0; r < job.n_runs; r++) {
            if (job.runs[r].n > 0 && job.runs[r].entries == nullptr) return LSM_ERR_NULL;
            if ((reinterpret_cast<uintptr_t>(job.runs[r].entries) & 63) != 0) return LSM_ERR_BAD_ARG;
            total += job.runs[r].n;
        }
        if (job.out.n_out == nullptr || (total > 0 && job.out.entries == nullptr)) return LSM_ERR_NULL;
        if ((reinterpret_cast<uintptr_t>(job.out.entries) & 63) != 0) return LSM_ERR_BAD_ARG;
        if (job.out.capacity < total) return LSM_ERR_CAPACITY;
    }
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < l.total) return LSM_ERR_WORKSPACE;
    // the host's table is built in pinned host memory kept per thread (so the copy below really is asynchronous) and
    // is not written again before the copy of the previous call from this thread has finished
    static thread_local BatchStaging staging;
    const size_t table_bytes = l.total - l.tile_job;
    unsigned char* table = staging.acquire(table_bytes);
    if (table == nullptr) return LSM_ERR_HIP;
    memset(table, 0, table_bytes);
    uint32_t* tile_job = reinterpret_cast<uint32_t*>(table);
    JobDesc* desc = reinterpret_cast<JobDesc*>(table + (l.jobs - l.tile_job));
    const lsm_entry_t** run_ptr = reinterpret_cast<const lsm_entry_t**>(table + (l.run_ptr - l.tile_job));
    uint64_t* run_n = reinterpret_cast<uint64_t*>(table + (l.run_n - l.tile_job));
    uint64_t tile = 0, split_word = 0, run = 0;
    bool any_fences = false;
    for (uint32_t j = 0; j < n_jobs; j++) {
        const lsm_compact_job_t& job = jobs[j];
        uint64_t total = 0;
        for (uint32_t r = 0; r < job.n_runs; r++) {
            run_ptr[run + r] = job.runs[r].entries;
            run_n[run + r] = job.runs[r].n;
            total += job.runs[r].n;
        }
        uint64_t nt = tiles_for(total, job.n_runs);
        if (nt == 0) nt = 1;
        JobDesc& d = desc[j];
        d.first_tile = tile;
        d.run_off = run;
        d.splits_off = split_word;
        d.out = job.out.entries;
        d.n_out = job.out.n_out;
        d.fence_out = reinterpret_cast<uint4*>(job.out.fence_keys);
        d.fence_stride = job.out.fence_keys ? job.out.fence_stride : 1u;
        any_fences = any_fences || job.out.fence_keys != nullptr;
        d.n_tiles = (uint32_t)nt;
        d.k = job.n_runs;
        d.flags = job.flags;
        for (uint64_t t = 0; t < nt; t++) tile_job[tile + t] = j;
        tile += nt;
        split_word += (nt + 1) * job.n_runs;
        run += job.n_runs;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    char* base = static_cast<char*>(workspace);
    if (hipMemcpyAsync(base + l.tile_job, table, table_bytes, hipMemcpyHostToDevice, stream) != hipSuccess) return LSM_ERR_HIP;
    if (!staging.copy_enqueued(stream)) return LSM_ERR_HIP;
    Workspace ws = {};
    ws.status = reinterpret_cast<uint64_t*>(base + l.status);
    ws.splits = reinterpret_cast<uint64_t*>(base + l.splits);
    ModeArgs ma = {};
    ma.tile_job = reinterpret_cast<const uint32_t*>(base + l.tile_job);
    ma.jobs = reinterpret_cast<const JobDesc*>(base + l.jobs);
    ma.run_ptr = reinterpret_cast<const lsm_entry_t* const*>(base + l.run_ptr);
    ma.run_n = reinterpret_cast<const uint64_t*>(base + l.run_n);
    int group = 1;
    while (group < (int)l.k_max) group <<= 1;
    const uint64_t per_block = (uint64_t)(256 / kWave) * (kWave / group);
    hipLaunchKernelGGL(partition_batch_kernel, dim3((uint32_t)((l.tiles + per_block - 1) / per_block)), dim3(256), 0, stream, ws, ma, l.tiles, group);
    RunTable rt = {};
    rt.k = 1;
    if (any_fences)  // the form that also writes fence indices (a job without one has a null pointer in its descriptor)
        hipLaunchKernelGGL((merge_kernel<1, kModeBatch>), dim3((uint32_t)l.tiles), dim3(kMergeThreads), 0, stream, rt, ws, l.tiles, 0u,
                           (lsm_entry_t*)nullptr, (uint64_t*)nullptr, (const uint64_t*)nullptr, 0u, (uint4*)nullptr, 1u, ma);
    else
        hipLaunchKernelGGL((merge_kernel<0, kModeBatch>), dim3((uint32_t)l.tiles), dim3(kMergeThreads), 0, stream, rt, ws, l.tiles, 0u,
                           (lsm_entry_t*)nullptr, (uint64_t*)nullptr, (const uint64_t*)nullptr, 0u, (uint4*)nullptr, 1u, ma);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

// ---------------------------------------------------------------------------------------
// lsm_compact_static: the same compaction for callers that cannot allocate device memory.  The workspace is a
// file-scope device array; each GPU holds its own copy at its own address, looked up once per device.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[LSM_STATIC_SCRATCH_BYTES];

namespace lsm {
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_lock;
static void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` on device d, once known

// Device address of this GPU's copy of `scratch` (the array's name itself is only a host-side handle).
static int scratch_address(void** ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LSM_ERR_HIP;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return LSM_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return LSM_OK;
}
}  // namespace lsm

extern "C" int lsm_compact_static(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* stream) {
    if (runs == nullptr) return LSM_ERR_NULL;
    if (n_runs == 0 || n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    if (flags & LSM_VALIDATE) return LSM_ERR_BAD_ARG;  // validation copies a status word to the host and waits
    uint64_t lens[LSM_MAX_RUNS];
    for (uint32_t j = 0; j < n_runs; j++) lens[j] = runs[j].n;
    if (lsm_compact_workspace_bytes(lens, n_runs) > (size_t)LSM_STATIC_SCRATCH_BYTES) return LSM_ERR_STATIC_LIMIT;
    void* ws = nullptr;
    const int rc = lsm::scratch_address(&ws);
    if (rc != LSM_OK) return rc;
    // every word of the scratch that a call reads is written by that call's own kernels first (the tile status words are
    // cleared before the merge), so what the previous call left behind does not matter
    return lsm_compact_remap(runs, n_runs, flags, out, ws, LSM_STATIC_SCRATCH_BYTES, stream, nullptr, nullptr);
}
