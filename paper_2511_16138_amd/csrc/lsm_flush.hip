// lsm_flush_buffer: the write buffer as a sorted run (paper section 2.2: the in-memory buffer is flushed as a
// sorted run).  A write buffer holds a few thousand entries, so every entry is simply compared with every other:
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

// kPlace = false: winner flags; kPlace = true: output positions of the winners, the copy, the count
template <bool kPlace>
__global__ void __launch_bounds__(kFlushThreads) flush_kernel(const lsm_entry_t* buffer, uint32_t n, uint32_t* winner, lsm_entry_t* out,
                                                               uint64_t* n_out, uint4* fence_out, uint32_t fence_stride) {
    __shared__ FlushTile tile;
    const uint32_t i = blockIdx.x * kFlushThreads + threadIdx.x;
    const bool mine = i < n;
    const uint4* me = reinterpret_cast<const uint4*>(buffer + (mine ? i : 0));
    const Key key = key_from_raw(me[0], me[1]);
    const uint64_t seq = buffer[mine ? i : 0].seqno;
    bool alive = mine && (!kPlace || winner[i] != 0);
    uint32_t before = 0;  // surviving entries with a smaller key
    for (uint32_t t0 = 0; t0 < n; t0 += kFlushThreads) {
        const uint32_t j = t0 + threadIdx.x;
        if (j < n) {
            const uint4* e = reinterpret_cast<const uint4*>(buffer + j);
            tile.lo[threadIdx.x] = e[0];
            tile.hi[threadIdx.x] = e[1];
            tile.seq[threadIdx.x] = buffer[j].seqno;
            if (kPlace) tile.wins[threadIdx.x] = winner[j];
        }
        __syncthreads();
        const uint32_t count = min((uint32_t)kFlushThreads, n - t0);
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
        uint4* dst = reinterpret_cast<uint4*>(out + before);
        for (int part = 0; part < 4; part++) dst[part] = src[part];
        if (fence_out != nullptr && before % fence_stride == 0) {
            fence_out[(before / fence_stride) * 2] = src[0];
            fence_out[(before / fence_stride) * 2 + 1] = src[1];
        }
    }
    // survivors of this workgroup -> total (n_out was cleared by the first kernel's launch sequence)
    const uint64_t votes = __ballot(alive);
    if ((threadIdx.x & (kWave - 1)) == 0 && votes) atomicAdd(reinterpret_cast<unsigned long long*>(n_out), (unsigned long long)__popcll(votes));
}

__global__ void flush_clear_kernel(uint64_t* n_out) { *n_out = 0; }

}  // namespace lsm

extern "C" size_t lsm_flush_workspace_bytes(uint64_t n) { return n <= LSM_MAX_BUFFER ? (size_t)n * sizeof(uint32_t) : 0; }

extern "C" int lsm_flush_buffer(const lsm_entry_t* buffer, uint64_t n, const lsm_out_t* out, void* workspace, size_t workspace_bytes,
                                void* stream_v) {
    using namespace lsm;
    if (out == nullptr || out->n_out == nullptr) return LSM_ERR_NULL;
    if (n > 0 && (buffer == nullptr || out->entries == nullptr)) return LSM_ERR_NULL;
    if (n > LSM_MAX_BUFFER) return LSM_ERR_BAD_ARG;
    if ((reinterpret_cast<uintptr_t>(buffer) & 63) != 0 || (reinterpret_cast<uintptr_t>(out->entries) & 63) != 0) return LSM_ERR_BAD_ARG;
    if (out->fence_keys != nullptr && (out->fence_stride == 0 || (reinterpret_cast<uintptr_t>(out->fence_keys) & 15) != 0))
        return LSM_ERR_BAD_ARG;
    if (out->capacity < n) return LSM_ERR_CAPACITY;
    if (n > 0 && (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 3) != 0 || workspace_bytes < lsm_flush_workspace_bytes(n)))
        return LSM_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_v);
    hipLaunchKernelGGL(flush_clear_kernel, dim3(1), dim3(1), 0, stream, out->n_out);
    if (n > 0) {
        const uint32_t blocks = (uint32_t)((n + kFlushThreads - 1) / kFlushThreads);
        uint32_t* winner = static_cast<uint32_t*>(workspace);
        uint4* fence_out = reinterpret_cast<uint4*>(out->fence_keys);
        const uint32_t fence_stride = out->fence_keys ? out->fence_stride : 1u;
        hipLaunchKernelGGL(flush_kernel<false>, dim3(blocks), dim3(kFlushThreads), 0, stream, buffer, (uint32_t)n, winner, out->entries,
                           out->n_out, fence_out, fence_stride);
        hipLaunchKernelGGL(flush_kernel<true>, dim3(blocks), dim3(kFlushThreads), 0, stream, buffer, (uint32_t)n, winner, out->entries,
                           out->n_out, fence_out, fence_stride);
    }
    return hipGetLastError() == hipSuccess ? LSM_OK : LSM_ERR_HIP;
}
