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
// range hands out the slots of its buckets with counters in LDS and writes every byte of its range exactly once.
// Which keys of a crowded bucket are kept, and the order of the slots in a bucket, depend on the order the
// workgroup happens to see the hashes in: lookups give the same answers for every such table.
#include <hip/hip_runtime.h>

#include "lsm_common.h"
#include "lsm_partition.h"

namespace lsm {

// one workgroup per range of kRangeUnits buckets
__global__ void __launch_bounds__(kPartThreads) index_fill_kernel(const uint64_t* ranged, const uint32_t* ranged_pos, const unsigned long long* totals,
                                                                 const unsigned long long* cursors, uint32_t n_buckets, uint8_t* table) {
    __shared__ uint32_t count[kRangeUnits];
    __shared__ uint16_t first_tag[kRangeUnits];  // the first slot's tag waits here: its field also carries the crowded bit
    const uint32_t first_bucket = blockIdx.x * kRangeUnits;
    const uint32_t buckets = n_buckets - first_bucket < kRangeUnits ? n_buckets - first_bucket : kRangeUnits;
    for (uint32_t b = threadIdx.x; b < buckets; b += kPartThreads) count[b] = 0;
    __syncthreads();
    const uint64_t end = cursors[blockIdx.x], begin = end - totals[blockIdx.x];
    for (uint64_t i = begin + threadIdx.x; i < end; i += kPartThreads) {
        const uint64_t h = ranged[i];
        const uint32_t b = bloom_block(h, n_buckets) - first_bucket;  // inside this range by construction
        const uint32_t k = atomicAdd(&count[b], 1u);
        if (k >= kIndexSlots) continue;  // a crowded bucket keeps the first eight keys that arrive
        uint8_t* bucket = table + (uint64_t)(first_bucket + b) * 64;
        const uint16_t tag = (uint16_t)(h & kIndexTagMask);
        if (k == 0) first_tag[b] = tag;
        else reinterpret_cast<uint16_t*>(bucket)[k] = tag;
        reinterpret_cast<uint32_t*>(bucket + 16)[k] = ranged_pos[i];
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < buckets; b += kPartThreads) {
        const uint32_t c = count[b];
        uint8_t* bucket = table + (uint64_t)(first_bucket + b) * 64;
        uint16_t* tags = reinterpret_cast<uint16_t*>(bucket);
        uint32_t* pos = reinterpret_cast<uint32_t*>(bucket + 16);
        tags[0] = (uint16_t)((c > 0 ? first_tag[b] : 0) | (c > kIndexSlots ? 0x8000u : 0u));
        for (uint32_t k = c > 0 ? c : 1; k < kIndexSlots; k++) tags[k] = 0;
        for (uint32_t k = c; k < kIndexSlots; k++) pos[k] = kIndexNoEntry;
        reinterpret_cast<uint4*>(bucket)[3] = make_uint4(0, 0, 0, 0);
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
    hipLaunchKernelGGL(index_fill_kernel, dim3(l.n_ranges), dim3(kPartThreads), 0, stream, reinterpret_cast<const uint64_t*>(base + l.ranged),
                       reinterpret_cast<const uint32_t*>(base + l.ranged_pos), reinterpret_cast<const unsigned long long*>(base + l.totals),
                       reinterpret_cast<const unsigned long long*>(base + l.cursors), (uint32_t)n_buckets, static_cast<uint8_t*>(table_out));
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
