// lsm_build_bloom: blocked Bloom filter of a run (paper section 2.2 names Bloom filters as the structure that
// lets a lookup skip a run; appendix B uses point lookups in "Probe").  One thread per entry: hash the key,
// OR its six bits into the 16-byte block (two 64-bit atomics at most).  Bits only ever get set, so the result is the same for any order.
#include <hip/hip_runtime.h>

#include "lsm_common.h"
#include "lsm_partition.h"

namespace lsm {

__global__ void bloom_clear_kernel(uint4* blocks, uint64_t n_blocks) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_blocks; i += stride) blocks[i] = make_uint4(0, 0, 0, 0);
}

__global__ void bloom_insert_kernel(const lsm_entry_t* entries, uint64_t n, uint32_t* words, uint32_t n_blocks) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint4 mask;
        const uint32_t block = bloom_block(bloom_hash(load_key(entries + i), mask), n_blocks);
        // two 64-bit halves (little-endian: word 0 is the low half of the first)
        unsigned long long* w = reinterpret_cast<unsigned long long*>(words + (uint64_t)block * 4);
        const unsigned long long lo = ((unsigned long long)mask.y << 32) | mask.x, hi = ((unsigned long long)mask.w << 32) | mask.z;
        if (lo) atomicOr(w + 0, lo);
        if (hi) atomicOr(w + 1, hi);
    }
}

// The same two steps for up to kBloomBatch runs per launch (blockIdx.y = run), for the many small runs that a round of
// flushes into several trees produces.
constexpr uint32_t kBloomBatch = 64;
struct BloomJobs {
    const lsm_entry_t* entries[kBloomBatch];
    uint64_t n[kBloomBatch];
    uint32_t* words[kBloomBatch];
    uint32_t n_blocks[kBloomBatch];
};

__global__ void bloom_clear_batch_kernel(BloomJobs jobs) {
    uint4* blocks = reinterpret_cast<uint4*>(jobs.words[blockIdx.y]);
    const uint64_t n_blocks = jobs.n_blocks[blockIdx.y], stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_blocks; i += stride) blocks[i] = make_uint4(0, 0, 0, 0);
}

__global__ void bloom_insert_batch_kernel(BloomJobs jobs) {
    const lsm_entry_t* entries = jobs.entries[blockIdx.y];
    uint32_t* words = jobs.words[blockIdx.y];
    const uint64_t n = jobs.n[blockIdx.y], stride = (uint64_t)gridDim.x * blockDim.x;
    const uint32_t n_blocks = jobs.n_blocks[blockIdx.y];
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint4 mask;
        const uint32_t block = bloom_block(bloom_hash(load_key(entries + i), mask), n_blocks);
        unsigned long long* w = reinterpret_cast<unsigned long long*>(words + (uint64_t)block * 4);
        const unsigned long long lo = ((unsigned long long)mask.y << 32) | mask.x, hi = ((unsigned long long)mask.w << 32) | mask.z;
        if (lo) atomicOr(w + 0, lo);
        if (hi) atomicOr(w + 1, hi);
    }
}

// A filter of at most kBloomSmallBlocks blocks (64 KiB) is built by one workgroup in LDS and written out once: one
// launch and no global atomics, for the short runs of a tree's upper levels.  blockIdx.y = run.
constexpr uint32_t kBloomSmallBlocks = 4096;
constexpr uint64_t kBloomSmallKeys = 1u << 18;  // a longer run with so small a filter is left to the whole device
constexpr int kBloomSmallThreads = 1024;
__global__ void __launch_bounds__(kBloomSmallThreads) bloom_small_kernel(BloomJobs jobs) {
    __shared__ uint32_t f[kBloomSmallBlocks * 4];
    const lsm_entry_t* entries = jobs.entries[blockIdx.y];
    const uint64_t n = jobs.n[blockIdx.y];
    const uint32_t n_blocks = jobs.n_blocks[blockIdx.y];  // <= kBloomSmallBlocks (checked by the host)
    for (uint32_t w = threadIdx.x; w < n_blocks * 4; w += kBloomSmallThreads) f[w] = 0;
    __syncthreads();
    // four keys per thread and step, all read before the first is hashed: a short run is one or two round trips
    constexpr int kAhead = 4;
    for (uint64_t i0 = threadIdx.x; i0 < n; i0 += (uint64_t)kAhead * kBloomSmallThreads) {
        Key key[kAhead];
#pragma unroll
        for (int a = 0; a < kAhead; a++) {
            const uint64_t i = i0 + (uint64_t)a * kBloomSmallThreads;
            key[a] = load_key(entries + (i < n ? i : i0));
        }
#pragma unroll
        for (int a = 0; a < kAhead; a++) {
            if (i0 + (uint64_t)a * kBloomSmallThreads >= n) break;
            uint4 mask;
            const uint32_t block = bloom_block(bloom_hash(key[a], mask), n_blocks);
            if (mask.x) atomicOr(&f[block * 4 + 0], mask.x);
            if (mask.y) atomicOr(&f[block * 4 + 1], mask.y);
            if (mask.z) atomicOr(&f[block * 4 + 2], mask.z);
            if (mask.w) atomicOr(&f[block * 4 + 3], mask.w);
        }
    }
    __syncthreads();
    uint4* out = reinterpret_cast<uint4*>(jobs.words[blockIdx.y]);
    const uint4* src = reinterpret_cast<const uint4*>(f);
    for (uint32_t b = threadIdx.x; b < n_blocks; b += kBloomSmallThreads) out[b] = src[b];
}

// ---------------------------------------------------------------------------------------
// Filter of a long run without global atomics.  The atomic build above is bound by the rate of read-modify-write
// operations on scattered 8-byte words (two per key); this one moves the keys' 8-byte hashes instead: they are sorted
// by ranges of kBucketBlocks consecutive filter blocks ("buckets", 64 KiB; the passes of lsm_partition.h), then one
// workgroup per bucket builds the bucket's 64 KiB of filter in LDS from the bucket's hashes and writes it out once.
// The order of the hashes inside a bucket does not matter: bits are only ever set.
// ---------------------------------------------------------------------------------------
constexpr uint32_t kBucketBlocks = kRangeUnits;  // filter blocks per bucket (64 KiB of LDS)

__global__ void hash_keys_kernel(const lsm_entry_t* entries, uint64_t n, uint64_t* hashes) {
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) hashes[i] = bloom_key_hash(load_key(entries + i));
}

// one workgroup per bucket; after the scatter pass cursors[b] is the END of bucket b's hashes, totals[b] their number
__global__ void __launch_bounds__(kPartThreads) bucket_fill_kernel(const uint64_t* bucketed, const unsigned long long* totals,
                                                                  const unsigned long long* cursors, uint32_t n_blocks, uint4* filter) {
    __shared__ uint32_t f[kBucketBlocks * 4];
    const uint32_t bucket = blockIdx.x, first_block = bucket * kBucketBlocks;
    const uint32_t blocks = n_blocks - first_block < kBucketBlocks ? n_blocks - first_block : kBucketBlocks;
    for (uint32_t w = threadIdx.x; w < blocks * 4; w += kPartThreads) f[w] = 0;
    __syncthreads();
    const uint64_t end = cursors[bucket], begin = end - totals[bucket];
    for (uint64_t i = begin + threadIdx.x; i < end; i += kPartThreads) {
        const uint64_t h = bucketed[i];
        const uint4 mask = bloom_mask(h);
        const uint32_t at = (bloom_block(h, n_blocks) - first_block) * 4;  // inside this bucket by construction
        if (mask.x) atomicOr(&f[at + 0], mask.x);
        if (mask.y) atomicOr(&f[at + 1], mask.y);
        if (mask.z) atomicOr(&f[at + 2], mask.z);
        if (mask.w) atomicOr(&f[at + 3], mask.w);
    }
    __syncthreads();
    const uint4* src = reinterpret_cast<const uint4*>(f);
    for (uint32_t b = threadIdx.x; b < blocks; b += kPartThreads) filter[first_block + b] = src[b];
}

}  // namespace lsm

extern "C" size_t lsm_bloom_workspace_bytes(uint64_t n, uint64_t n_blocks) {
    if (!lsm::range_partition_applies(n, n_blocks)) return 0;
    return lsm::range_layout(n, n_blocks, false).total;
}

extern "C" int lsm_hash_keys(const lsm_run_t* run, uint64_t* hashes_out, void* stream_v) {
    using namespace lsm;
    if (run == nullptr) return LSM_ERR_NULL;
    if (run->n == 0) return LSM_OK;
    if (run->entries == nullptr || hashes_out == nullptr) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(run->entries) & 63) != 0 || (reinterpret_cast<uintptr_t>(hashes_out) & 7) != 0) return LSM_ERR_BAD_ARG;
    uint64_t blocks = (run->n + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(hash_keys_kernel, dim3((uint32_t)blocks), dim3(256), 0, static_cast<hipStream_t>(stream_v), run->entries, run->n, hashes_out);
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

extern "C" int lsm_build_bloom_hashed(const uint64_t* hashes, uint64_t n, void* filter_out, uint64_t n_blocks, void* workspace,
                                      size_t workspace_bytes, void* stream_v) {
    using namespace lsm;
    if (filter_out == nullptr || (n > 0 && hashes == nullptr)) return LSM_ERR_NULL;
    if (n_blocks == 0 || n_blocks >= (1ull << 32)) return LSM_ERR_BAD_ARG;
    if ((reinterpret_cast<uintptr_t>(filter_out) & 15) != 0 || (reinterpret_cast<uintptr_t>(hashes) & 7) != 0) return LSM_ERR_BAD_ARG;
    if (!range_partition_applies(n, n_blocks)) return LSM_ERR_BAD_ARG;
    const RangeLayout l = range_layout(n, n_blocks, false);
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < l.total) return LSM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    launch_range_partition<false>(hashes, n, n_blocks, l, workspace, stream);
    char* base = static_cast<char*>(workspace);
    const unsigned long long* totals = reinterpret_cast<const unsigned long long*>(base + l.totals);
    const unsigned long long* cursors = reinterpret_cast<const unsigned long long*>(base + l.cursors);
    const uint64_t* bucketed = reinterpret_cast<const uint64_t*>(base + l.ranged);
    hipLaunchKernelGGL(bucket_fill_kernel, dim3(l.n_ranges), dim3(kPartThreads), 0, stream, bucketed, totals, cursors, (uint32_t)n_blocks,
                       static_cast<uint4*>(filter_out));
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

extern "C" uint64_t lsm_bloom_blocks(uint64_t n, uint32_t bits_per_key) {
    if (bits_per_key == 0) return 0;
    const unsigned __int128 bits = (unsigned __int128)n * bits_per_key;
    const unsigned __int128 blocks = bits == 0 ? 1 : (bits + 127) / 128;
    return blocks >= ((unsigned __int128)1 << 32) ? 0 : (uint64_t)blocks;
}

extern "C" int lsm_build_bloom(const lsm_run_t* run, void* filter_out, uint64_t n_blocks, void* stream_v) {
    using namespace lsm;
    if (run == nullptr || filter_out == nullptr) return LSM_ERR_NULL;
    if (run->n > 0 && run->entries == nullptr) return LSM_ERR_NULL;
    if (n_blocks == 0 || n_blocks >= (1ull << 32)) return LSM_ERR_BAD_ARG;
    if ((reinterpret_cast<uintptr_t>(filter_out) & 15) != 0 || (reinterpret_cast<uintptr_t>(run->entries) & 63) != 0)
        return LSM_ERR_BAD_ARG;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    if (n_blocks <= kBloomSmallBlocks && run->n <= kBloomSmallKeys) {
        BloomJobs jobs = {};
        jobs.entries[0] = run->entries;
        jobs.n[0] = run->n;
        jobs.words[0] = static_cast<uint32_t*>(filter_out);
        jobs.n_blocks[0] = (uint32_t)n_blocks;
        hipLaunchKernelGGL(bloom_small_kernel, dim3(1, 1), dim3(kBloomSmallThreads), 0, stream, jobs);
        return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
    }
    uint64_t clear_blocks = (n_blocks + 255) / 256;
    if (clear_blocks > 4096) clear_blocks = 4096;
    hipLaunchKernelGGL(bloom_clear_kernel, dim3((uint32_t)clear_blocks), dim3(256), 0, stream, static_cast<uint4*>(filter_out), n_blocks);
    if (run->n > 0) {
        uint64_t blocks = (run->n + 255) / 256;
        if (blocks > 16384) blocks = 16384;
        hipLaunchKernelGGL(bloom_insert_kernel, dim3((uint32_t)blocks), dim3(256), 0, stream, run->entries, run->n,
                           static_cast<uint32_t*>(filter_out), (uint32_t)n_blocks);
    }
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}

extern "C" int lsm_build_bloom_batch(const lsm_run_t* runs, void* const* filters_out, const uint64_t* n_blocks, uint32_t n_runs,
                                     void* stream_v) {
    using namespace lsm;
    if (n_runs == 0) return LSM_OK;
    if (runs == nullptr || filters_out == nullptr || n_blocks == nullptr) return LSM_ERR_NULL;
    for (uint32_t j = 0; j < n_runs; j++) {
        if (filters_out[j] == nullptr || (runs[j].n > 0 && runs[j].entries == nullptr)) return LSM_ERR_NULL;
        if (n_blocks[j] == 0 || n_blocks[j] >= (1ull << 32)) return LSM_ERR_BAD_ARG;
        if ((reinterpret_cast<uintptr_t>(filters_out[j]) & 15) != 0 || (reinterpret_cast<uintptr_t>(runs[j].entries) & 63) != 0)
            return LSM_ERR_BAD_ARG;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    for (uint32_t first = 0; first < n_runs; first += kBloomBatch) {
        const uint32_t count = n_runs - first < kBloomBatch ? n_runs - first : kBloomBatch;
        BloomJobs jobs = {};
        uint64_t most_blocks = 1, most_entries = 0;
        for (uint32_t j = 0; j < count; j++) {
            jobs.entries[j] = runs[first + j].entries;
            jobs.n[j] = runs[first + j].n;
            jobs.words[j] = static_cast<uint32_t*>(filters_out[first + j]);
            jobs.n_blocks[j] = (uint32_t)n_blocks[first + j];
            most_blocks = n_blocks[first + j] > most_blocks ? n_blocks[first + j] : most_blocks;
            most_entries = runs[first + j].n > most_entries ? runs[first + j].n : most_entries;
        }
        if (most_blocks <= kBloomSmallBlocks && most_entries <= kBloomSmallKeys) {
            hipLaunchKernelGGL(bloom_small_kernel, dim3(1, count), dim3(kBloomSmallThreads), 0, stream, jobs);
            continue;
        }
        uint64_t cx = (most_blocks + 255) / 256, ix = (most_entries + 255) / 256;
        if (cx > 1024) cx = 1024;
        if (ix > 4096) ix = 4096;
        hipLaunchKernelGGL(bloom_clear_batch_kernel, dim3((uint32_t)cx, count), dim3(256), 0, stream, jobs);
        if (most_entries > 0) hipLaunchKernelGGL(bloom_insert_batch_kernel, dim3((uint32_t)ix, count), dim3(256), 0, stream, jobs);
    }
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
