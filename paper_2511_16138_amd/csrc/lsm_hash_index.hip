// lsm_build_hash_index: hash index of a run.  Paper section 2.2 has a point lookup go through a Bloom filter and the
// in-memory fence pointers of a run; with the run in HBM the fence search is a dozen dependent reads.  This index
// answers "can the key be in this run, and where" with one 16-byte read (the tags of the key's bucket) and finds
// the entry with one more read of the same 64-byte line: it does the work of the filter (a key whose tag is not in
// its bucket is not in the run) and of the fence search.
//
// Format (also in the header, at lsm_hash_index_t): ceil(n / 4) buckets of 64 bytes with eight slots; a key with filter
// hash h belongs to bucket ((h >> 32) * n_buckets) >> 32 and has the 15-bit tag h & 0x7FFF.  Bytes 0..15 of a bucket
// are the slots' tag fields (16 bits each), bytes 16..47 the slots' positions in the run (32 bits each, all ones = empty
// slot), the rest is zero.  A bucket that more than eight keys fall into holds eight of them and has bit 15 of its
// first tag field set, which sends a lookup that finds nothing among the eight to the fence index.
//
// Build: the hashes and their positions are sorted by ranges of 4,096 buckets (lsm_partition.h); one workgroup per
// range hands out the slots of its buckets with counters in LDS, assembles the buckets there, and writes every byte of
// its range exactly once.
// Which keys of a crowded bucket are kept, and the order of the slots in a bucket, depend on the order the
// workgroup happens to see the hashes in: lookups give the same answers for every such table.
#include <hip/hip_runtime.h>

#include "lsm_common.h"
#include "lsm_partition.h"

namespace lsm {

// One workgroup per range of kRangeUnits buckets.  The range is built a quarter at a time in LDS (1,024 buckets = 64 KiB)
// and each quarter leaves with contiguous 16-byte stores: scattered 2- and 4-byte stores straight into the table cost
// 4.6 bytes of HBM writes per byte of table.  Every pass reads the range's hashes again (they stay in the caches).
constexpr uint32_t kFillBuckets = 1024;
__global__ void __launch_bounds__(kPartThreads) index_fill_kernel(const uint4* ranged, const unsigned long long* totals,
                                                                 const unsigned long long* cursors, uint32_t n_buckets, uint4* table) {
    __shared__ uint4 part[kFillBuckets * 4];  // the buckets of this pass
    __shared__ uint32_t count[kFillBuckets];
    const uint32_t range_first = blockIdx.x * kRangeUnits;
    const uint64_t end = cursors[blockIdx.x], begin = end - totals[blockIdx.x];
    for (uint32_t first_bucket = range_first; first_bucket < range_first + kRangeUnits && first_bucket < n_buckets; first_bucket += kFillBuckets) {
        const uint32_t buckets = n_buckets - first_bucket < kFillBuckets ? n_buckets - first_bucket : kFillBuckets;
        // every bucket starts empty: tag fields 0, positions all ones, the rest 0
        for (uint32_t i = threadIdx.x; i < buckets * 4; i += kPartThreads) {
            const uint32_t fill = ((i & 3) == 1 || (i & 3) == 2) ? kIndexNoEntry : 0u;
            part[i] = make_uint4(fill, fill, fill, fill);
        }
        for (uint32_t b = threadIdx.x; b < buckets; b += kPartThreads) count[b] = 0;
        __syncthreads();
        uint16_t* tags = reinterpret_cast<uint16_t*>(part);
        uint32_t* words = reinterpret_cast<uint32_t*>(part);
        for (uint64_t i = begin + threadIdx.x; i < end; i += kPartThreads) {
            const uint4 rec = ranged[i];  // {h, position, 0}
            const uint64_t h = ((uint64_t)rec.y << 32) | rec.x;
            const uint32_t b = bloom_block(h, n_buckets) - first_bucket;  // wraps for the buckets before this pass
            if (b >= buckets) continue;
            const uint32_t k = atomicAdd(&count[b], 1u);
            if (k >= kIndexSlots) continue;  // a crowded bucket keeps the first eight keys that arrive
            tags[b * 32 + k] = (uint16_t)(h & kIndexTagMask);
            words[b * 16 + 4 + k] = rec.z;
        }
        __syncthreads();
        for (uint32_t b = threadIdx.x; b < buckets; b += kPartThreads)
            if (count[b] > kIndexSlots) tags[b * 32] |= 0x8000u;  // crowded
        __syncthreads();
        uint4* dst = table + (uint64_t)first_bucket * 4;
        for (uint32_t i = threadIdx.x; i < buckets * 4; i += kPartThreads) dst[i] = part[i];
        __syncthreads();  // the LDS arrays are reused by the next pass
    }
}

}  // namespace lsm

extern "C" uint64_t lsm_hash_index_buckets(uint64_t n) { return lsm::index_buckets(n); }

extern "C" size_t lsm_hash_index_workspace_bytes(uint64_t n) {
    if (n >= 0xFFFFFFFFull || !lsm::range_partition_applies(n, lsm::index_buckets(n))) return 0;
    return lsm::range_layout(n, lsm::index_buckets(n), true).total;
}

extern "C" int lsm_build_hash_index(const uint64_t* hashes, uint64_t n, void* table_out, void* workspace, size_t workspace_bytes,
                                    void* stream_v) {
    using namespace lsm;
    if (table_out == nullptr || (n > 0 && hashes == nullptr)) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(table_out) & 63) != 0 || (reinterpret_cast<uintptr_t>(hashes) & 7) != 0) return LSM_ERR_BAD_ARG;
    const uint64_t n_buckets = index_buckets(n);
    if (n >= 0xFFFFFFFFull || !range_partition_applies(n, n_buckets)) return LSM_ERR_BAD_ARG;  // positions are 32-bit, all ones = no entry
    const RangeLayout l = range_layout(n, n_buckets, true);
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255) != 0 || workspace_bytes < l.total) return LSM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    launch_range_partition<true>(hashes, n, n_buckets, l, workspace, stream);
    char* base = static_cast<char*>(workspace);
    hipLaunchKernelGGL(index_fill_kernel, dim3(l.n_ranges), dim3(kPartThreads), 0, stream, reinterpret_cast<const uint4*>(base + l.ranged),
                       reinterpret_cast<const unsigned long long*>(base + l.totals),
                       reinterpret_cast<const unsigned long long*>(base + l.cursors), (uint32_t)n_buckets, static_cast<uint4*>(table_out));
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
