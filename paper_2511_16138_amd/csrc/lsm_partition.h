// Sorting key hashes by where they land in a hashed structure (Bloom filter blocks, hash index buckets), so that the
// structure can be built range by range in on-chip memory instead of by read-modify-write operations on scattered
// words of HBM.  A hash's unit (filter block, index bucket) is ((h >> 32) * n_units) >> 32, which grows with the hash,
// so a range of kRangeUnits consecutive units is a contiguous range of hash values.
//   count     every workgroup counts, in LDS, how many hashes of its chunk fall into each range and adds its counts to
//             the range totals (one global atomic per range and workgroup)
//   offsets   exclusive prefix sum over the range totals (one workgroup)
//   scatter   every workgroup counts its chunk again, reserves its share of each range with one returning atomic per
//             range, and copies each hash (with its position in the input, if asked) to its range's part of the
//             workspace; afterwards cursors[r] is the END of range r's hashes and totals[r] their number
// The order of the hashes inside a range is not defined.
#ifndef LSM_PARTITION_H
#define LSM_PARTITION_H

#include <hip/hip_runtime.h>

#include "lsm_common.h"

namespace lsm {

constexpr uint32_t kRangeUnits = 4096;    // units (filter blocks, index buckets) per range
constexpr uint32_t kMaxRanges = 8192;     // range counters of a workgroup (32 KiB of LDS)
constexpr uint32_t kChunkHashes = 65536;  // hashes per workgroup of the count and scatter passes
constexpr int kPartThreads = 1024;

static __global__ void range_clear_kernel(uint64_t* totals, uint32_t n_ranges) {
    for (uint32_t b = blockIdx.x * blockDim.x + threadIdx.x; b < n_ranges; b += gridDim.x * blockDim.x) totals[b] = 0;
}

// kScatter = false: count.  kScatter = true: count, reserve, copy.  kWithPos: the copy of hash i is a 16-byte record
// {h, i, 0}: one store per hash (an 8-byte and a 4-byte store into two arrays took a fifth longer).
template <bool kScatter, bool kWithPos>
__global__ void __launch_bounds__(kPartThreads) range_pass_kernel(const uint64_t* hashes, uint64_t n, uint32_t n_units, uint32_t n_ranges,
                                                                 unsigned long long* totals, unsigned long long* cursors, uint64_t* ranged) {
    __shared__ uint32_t count[kMaxRanges];
    const uint64_t first = (uint64_t)blockIdx.x * kChunkHashes;
    const uint64_t last = first + kChunkHashes < n ? first + kChunkHashes : n;
    for (uint32_t b = threadIdx.x; b < n_ranges; b += kPartThreads) count[b] = 0;
    __syncthreads();
    for (uint64_t i = first + threadIdx.x; i < last; i += kPartThreads) atomicAdd(&count[bloom_block(hashes[i], n_units) / kRangeUnits], 1u);
    __syncthreads();
    if (!kScatter) {
        for (uint32_t b = threadIdx.x; b < n_ranges; b += kPartThreads)
            if (count[b]) atomicAdd(&totals[b], (unsigned long long)count[b]);
        return;
    }
    // count[b] becomes where this workgroup's next hash of range b goes (the workspace holds fewer than 2^32 hashes)
    for (uint32_t b = threadIdx.x; b < n_ranges; b += kPartThreads)
        if (count[b]) count[b] = (uint32_t)atomicAdd(&cursors[b], (unsigned long long)count[b]);
    __syncthreads();
    for (uint64_t i = first + threadIdx.x; i < last; i += kPartThreads) {
        const uint64_t h = hashes[i];
        const uint32_t at = atomicAdd(&count[bloom_block(h, n_units) / kRangeUnits], 1u);
        if (kWithPos) reinterpret_cast<uint4*>(ranged)[at] = make_uint4((uint32_t)h, (uint32_t)(h >> 32), (uint32_t)i, 0);  // one 16-byte record
        else ranged[at] = h;
    }
}

// cursors[b] = number of hashes in the ranges before b (one workgroup); totals[b] keeps the range's own count
static __global__ void __launch_bounds__(kPartThreads) range_offsets_kernel(const unsigned long long* totals, unsigned long long* cursors,
                                                                           uint32_t n_ranges) {
    __shared__ unsigned long long wave_sum[kPartThreads / kWave];
    constexpr uint32_t kPer = kMaxRanges / kPartThreads;  // consecutive ranges per thread
    unsigned long long v[kPer], mine = 0;
    for (uint32_t i = 0; i < kPer; i++) {
        const uint32_t b = threadIdx.x * kPer + i;
        v[i] = b < n_ranges ? totals[b] : 0;
        mine += v[i];
    }
    unsigned long long incl = mine;
    const int lane = threadIdx.x & (kWave - 1);
    for (int off = 1; off < kWave; off <<= 1) {
        const unsigned long long o = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += o;
    }
    if (lane == kWave - 1) wave_sum[threadIdx.x / kWave] = incl;
    __syncthreads();
    unsigned long long before = incl - mine;
    for (uint32_t w = 0; w < threadIdx.x / kWave; w++) before += wave_sum[w];
    for (uint32_t i = 0; i < kPer; i++) {
        const uint32_t b = threadIdx.x * kPer + i;
        if (b < n_ranges) cursors[b] = before;
        before += v[i];
    }
}

// Workspace of a partition of n hashes into n_ranges ranges: totals, cursors, the hashes (or records) by range.
struct RangeLayout {
    uint32_t n_ranges;
    size_t totals, cursors, ranged, total;
};
inline RangeLayout range_layout(uint64_t n, uint64_t n_units, bool with_pos) {
    auto up = [](size_t x) { return (x + 255) & ~size_t(255); };
    RangeLayout l;
    l.n_ranges = (uint32_t)((n_units + kRangeUnits - 1) / kRangeUnits);
    l.totals = 0;
    l.cursors = l.totals + up((size_t)l.n_ranges * 8);
    l.ranged = l.cursors + up((size_t)l.n_ranges * 8);
    l.total = l.ranged + up((size_t)n * (with_pos ? 16 : 8));
    return l;
}
inline bool range_partition_applies(uint64_t n, uint64_t n_units) {
    return n_units > 0 && n < (1ull << 32) && (n_units + kRangeUnits - 1) / kRangeUnits <= kMaxRanges;
}

// Enqueues the four passes.  `workspace` is laid out by range_layout.
template <bool kWithPos>
inline void launch_range_partition(const uint64_t* hashes, uint64_t n, uint64_t n_units, const RangeLayout& l, void* workspace, hipStream_t stream) {
    char* base = static_cast<char*>(workspace);
    unsigned long long* totals = reinterpret_cast<unsigned long long*>(base + l.totals);
    unsigned long long* cursors = reinterpret_cast<unsigned long long*>(base + l.cursors);
    uint64_t* ranged = reinterpret_cast<uint64_t*>(base + l.ranged);
    const uint32_t chunks = (uint32_t)((n + kChunkHashes - 1) / kChunkHashes);
    hipLaunchKernelGGL(range_clear_kernel, dim3((l.n_ranges + 255) / 256), dim3(256), 0, stream, reinterpret_cast<uint64_t*>(totals), l.n_ranges);
    if (chunks > 0)
        hipLaunchKernelGGL((range_pass_kernel<false, kWithPos>), dim3(chunks), dim3(kPartThreads), 0, stream, hashes, n, (uint32_t)n_units, l.n_ranges,
                           totals, cursors, ranged);
    hipLaunchKernelGGL(range_offsets_kernel, dim3(1), dim3(kPartThreads), 0, stream, totals, cursors, l.n_ranges);
    if (chunks > 0)
        hipLaunchKernelGGL((range_pass_kernel<true, kWithPos>), dim3(chunks), dim3(kPartThreads), 0, stream, hashes, n, (uint32_t)n_units, l.n_ranges,
                           totals, cursors, ranged);
}

}  // namespace lsm

#endif
