// lsm_flush_buffer: the write buffer as a sorted run (paper section 2.2: the in-memory buffer is flushed as a
// sorted run).  A buffer of a few thousand entries is sorted by comparing every entry with every other; a larger one is
// cut into segments of kFlushSegment entries in write order, every segment is sorted that way (all segments in one
// launch), and the sorted segments are merged by the compaction kernels (the segment written last is the newest run,
// so that among equal sequence numbers the later write wins there as well).  The all-pairs step:
//   winner_kernel  entry i survives unless some entry j has the same key and is newer (larger seqno, or the same
//                  seqno and written later);
//   place_kernel   a surviving entry goes to position |{surviving j : key_j < key_i}|; the survivors are counted.
// Both kernels stream the whole buffer through LDS in tiles (key + seqno, and the winner flag in the second),
// and all threads of a workgroup read the same tile record at the same time (LDS broadcast).
#include <hip/hip_runtime.h>

#include "lsm_common.h"

namespace lsm {

constexpr int kFlushThreads = 256;

struct FlushTile {
    uint4 lo[kFlushThreads];   // key bytes 0..15
    uint4 hi[kFlushThreads];   // key bytes 16..31
    uint64_t seq[kFlushThreads];
    uint32_t wins[kFlushThreads];
};

__device__ __forceinline__ int key_cmp(const Key& a, const Key& b) {
    for (int w = 0; w < 4; w++)
        if (a.w[w] != b.w[w]) return a.w[w] < b.w[w] ? -1 : 1;
    return 0;
}

// kPlace = false: winner flags; kPlace = true: output positions of the winners, the copy, the count.
// blockIdx.y = segment: the entries [y * segment, min(n, (y + 1) * segment)) are sorted among themselves, written to
// out + y * segment, and counted in n_out[y] (one segment that is the whole buffer: the plain case).
template <bool kPlace>
__global__ void __launch_bounds__(kFlushThreads) flush_kernel(const lsm_entry_t* buffer, uint32_t n, uint32_t segment, uint32_t* winner,
                                                               lsm_entry_t* out, uint64_t* n_out, uint4* fence_out, uint32_t fence_stride) {
    __shared__ FlushTile tile;
    const uint32_t seg_lo = blockIdx.y * segment, seg_hi = min(n, seg_lo + segment);
    const uint32_t i = seg_lo + blockIdx.x * kFlushThreads + threadIdx.x;
    const bool mine = i < seg_hi;
    const uint4* me = reinterpret_cast<const uint4*>(buffer + (mine ? i : seg_lo));
    const Key key = key_from_raw(me[0], me[1]);
    const uint64_t seq = buffer[mine ? i : seg_lo].seqno;
    bool alive = mine && (!kPlace || winner[i] != 0);
    uint32_t before = 0;  // surviving entries of the segment with a smaller key
    for (uint32_t t0 = seg_lo; t0 < seg_hi; t0 += kFlushThreads) {
        const uint32_t j = t0 + threadIdx.x;
        if (j < seg_hi) {
            const uint4* e = reinterpret_cast<const uint4*>(buffer + j);
            tile.lo[threadIdx.x] = e[0];
            tile.hi[threadIdx.x] = e[1];
            tile.seq[threadIdx.x] = buffer[j].seqno;
            if (kPlace) tile.wins[threadIdx.x] = winner[j];
        }
        __syncthreads();
        const uint32_t count = min((uint32_t)kFlushThreads, seg_hi - t0);
        if (alive) {
            for (uint32_t c = 0; c < count; c++) {
                const int cmp = key_cmp(key_from_raw(tile.lo[c], tile.hi[c]), key);
                if (kPlace) {
                    before += (cmp < 0 && tile.wins[c]) ? 1 : 0;
                } else if (cmp == 0) {
                    const uint64_t other = tile.seq[c];
                    if (other > seq || (other == seq && t0 + c > i)) alive = false;  // a newer version of the same key
                }
            }
        }
        __syncthreads();
    }
    if (!kPlace) {
        if (mine) winner[i] = alive ? 1 : 0;
        return;
    }
    if (alive) {
        const uint4* src = reinterpret_cast<const uint4*>(buffer + i);
        uint4* dst = reinterpret_cast<uint4*>(out + seg_lo + before);
        for (int part = 0; part < 4; part++) dst[part] = src[part];
        if (fence_out != nullptr && before % fence_stride == 0) {
            fence_out[(before / fence_stride) * 2] = src[0];
            fence_out[(before / fence_stride) * 2 + 1] = src[1];
        }
    }
    // survivors of this workgroup -> the segment's total (cleared by flush_clear_kernel)
    const uint64_t votes = __ballot(alive);
    if ((threadIdx.x & (kWave - 1)) == 0 && votes)
        atomicAdd(reinterpret_cast<unsigned long long*>(n_out + blockIdx.y), (unsigned long long)__popcll(votes));
}

__global__ void flush_clear_kernel(uint64_t* n_out, uint32_t count) {
    if (threadIdx.x < count) n_out[threadIdx.x] = 0;
}

constexpr uint64_t kFlushDirect = 8192;    // up to here one all-pairs sort of the whole buffer
constexpr uint64_t kFlushSegment = 4096;   // beyond: segments of this many entries, then one merge of the segments
static_assert(kFlushSegment * LSM_MAX_RUNS >= LSM_MAX_BUFFER, "the segments of the largest buffer must fit one compaction");

__host__ inline size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

// Workspace of the segmented path: sorted segments | winner flags | segment counts | compaction workspace.
struct FlushLayout {
    size_t sorted, winner, counts, compact, total;
    uint32_t segments;
    uint64_t upper[LSM_MAX_RUNS];  // entries per segment, newest segment first (the order the compaction takes them in)
};
static FlushLayout flush_layout(uint64_t n) {
    FlushLayout l;
    l.segments = (uint32_t)((n + kFlushSegment - 1) / kFlushSegment);
    for (uint32_t j = 0; j < LSM_MAX_RUNS; j++) l.upper[j] = 0;
    for (uint32_t g = 0; g < l.segments; g++) {
        const uint64_t lo = g * kFlushSegment;
        l.upper[l.segments - 1 - g] = (n - lo < kFlushSegment) ? n - lo : kFlushSegment;
    }
    l.sorted = 0;
    l.winner = up256(n * sizeof(lsm_entry_t));
    l.counts = l.winner + up256(n * sizeof(uint32_t));
    l.compact = l.counts + up256(2 * LSM_MAX_RUNS * sizeof(uint64_t));
    l.total = l.compact + lsm_compact_workspace_bytes(l.upper, l.segments);
    return l;
}

// counts of the segments in write order -> the same counts in the order of the compaction's runs (newest first)
__global__ void flush_reverse_counts_kernel(const uint64_t* in, uint64_t* out, uint32_t segments) {
    if (threadIdx.x < segments) out[threadIdx.x] = in[segments - 1 - threadIdx.x];
}

}  // namespace lsm

extern "C" size_t lsm_flush_workspace_bytes(uint64_t n) {
    if (n > LSM_MAX_BUFFER) return 0;
    return n <= lsm::kFlushDirect ? (size_t)n * sizeof(uint32_t) : lsm::flush_layout(n).total;
}

extern "C" int lsm_flush_buffer(const lsm_entry_t* buffer, uint64_t n, const lsm_out_t* out, void* workspace, size_t workspace_bytes,
                                void* stream_v) {
    using namespace lsm;
    if (out == nullptr || out->n_out == nullptr) return LSM_ERR_NULL;
    if (n > 0 && (buffer == nullptr || out->entries == nullptr)) return LSM_ERR_NULL;
    if (n > LSM_MAX_BUFFER) return LSM_ERR_BAD_ARG;
    if ((reinterpret_cast<uintptr_t>(buffer) & 63) != 0 || (reinterpret_cast<uintptr_t>(out->entries) & 63) != 0) return LSM_ERR_BAD_ARG;
    if (out->fence_keys != nullptr && (out->fence_stride == 0 || (reinterpret_cast<uintptr_t>(out->fence_keys) & 15) != 0))
        return LSM_ERR_BAD_ARG;
    if (out->key_hashes != nullptr) return LSM_ERR_BAD_ARG;  // the filter of a flushed run: lsm_build_bloom
    if (out->capacity < n) return LSM_ERR_CAPACITY;
    const bool direct = n <= kFlushDirect;
    if (n > 0 && (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & (direct ? 3 : 255)) != 0 ||
                  workspace_bytes < lsm_flush_workspace_bytes(n)))
        return LSM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    uint4* fence_out = reinterpret_cast<uint4*>(out->fence_keys);
    const uint32_t fence_stride = out->fence_keys ? out->fence_stride : 1u;
    if (direct) {
        hipLaunchKernelGGL(flush_clear_kernel, dim3(1), dim3(64), 0, stream, out->n_out, 1u);
        if (n > 0) {
            const uint32_t blocks = (uint32_t)((n + kFlushThreads - 1) / kFlushThreads);
            uint32_t* winner = static_cast<uint32_t*>(workspace);
            hipLaunchKernelGGL(flush_kernel<false>, dim3(blocks), dim3(kFlushThreads), 0, stream, buffer, (uint32_t)n, (uint32_t)n, winner,
                               out->entries, out->n_out, fence_out, fence_stride);
            hipLaunchKernelGGL(flush_kernel<true>, dim3(blocks), dim3(kFlushThreads), 0, stream, buffer, (uint32_t)n, (uint32_t)n, winner,
                               out->entries, out->n_out, fence_out, fence_stride);
        }
        return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
    }
    // segments sorted on their own, into the workspace
    const FlushLayout l = flush_layout(n);
    char* base = static_cast<char*>(workspace);
    lsm_entry_t* sorted = reinterpret_cast<lsm_entry_t*>(base + l.sorted);
    uint32_t* winner = reinterpret_cast<uint32_t*>(base + l.winner);
    uint64_t* counts = reinterpret_cast<uint64_t*>(base + l.counts);  // [segments] in write order, then [segments] newest first
    hipLaunchKernelGGL(flush_clear_kernel, dim3(1), dim3(64), 0, stream, counts, l.segments);
    const dim3 grid((uint32_t)(kFlushSegment / kFlushThreads), l.segments);
    hipLaunchKernelGGL(flush_kernel<false>, grid, dim3(kFlushThreads), 0, stream, buffer, (uint32_t)n, (uint32_t)kFlushSegment, winner, sorted,
                       counts, (uint4*)nullptr, 1u);
    hipLaunchKernelGGL(flush_kernel<true>, grid, dim3(kFlushThreads), 0, stream, buffer, (uint32_t)n, (uint32_t)kFlushSegment, winner, sorted,
                       counts, (uint4*)nullptr, 1u);
    hipLaunchKernelGGL(flush_reverse_counts_kernel, dim3(1), dim3(64), 0, stream, counts, counts + LSM_MAX_RUNS, l.segments);
    if (hipGetLastError() != hipSuccess) return LSM_ERR_HIP;
    // one merge of the sorted segments, the one written last first; their lengths stay on the device
    const lsm_entry_t* ptr[LSM_MAX_RUNS];
    for (uint32_t j = 0; j < l.segments; j++) ptr[j] = sorted + (uint64_t)(l.segments - 1 - j) * kFlushSegment;
    return compact_device_lengths(ptr, l.upper, counts + LSM_MAX_RUNS, l.segments, 0, out, base + l.compact, workspace_bytes - l.compact, stream);
}
