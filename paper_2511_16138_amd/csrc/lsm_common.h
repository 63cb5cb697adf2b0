// Shared device-side definitions of the LSM key-index kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lsm_index.h"

namespace lsm {

constexpr int kWave = 64;

// A key as four big-endian-numeric words: comparing w[0], w[1], ... as unsigned integers is
// byte-string (memcmp) order of the 32 key bytes.
struct Key {
    uint64_t w[4];
};

__device__ __forceinline__ Key key_from_raw(uint4 lo, uint4 hi) {
    Key k;
    k.w[0] = __builtin_bswap64(((uint64_t)lo.y << 32) | lo.x);
    k.w[1] = __builtin_bswap64(((uint64_t)lo.w << 32) | lo.z);
    k.w[2] = __builtin_bswap64(((uint64_t)hi.y << 32) | hi.x);
    k.w[3] = __builtin_bswap64(((uint64_t)hi.w << 32) | hi.z);
    return k;
}

// Key of an entry (or of a 32-byte key record) in global or shared memory; p is 16-byte aligned.
__device__ __forceinline__ Key load_key(const void* p) {
    const uint4* q = reinterpret_cast<const uint4*>(p);
    return key_from_raw(q[0], q[1]);
}

__device__ __forceinline__ bool key_less(const Key& a, const Key& b) {
    if (a.w[0] != b.w[0]) return a.w[0] < b.w[0];
    if (a.w[1] != b.w[1]) return a.w[1] < b.w[1];
    if (a.w[2] != b.w[2]) return a.w[2] < b.w[2];
    return a.w[3] < b.w[3];
}

__device__ __forceinline__ bool key_equal(const Key& a, const Key& b) {
    return ((a.w[0] ^ b.w[0]) | (a.w[1] ^ b.w[1]) | (a.w[2] ^ b.w[2]) | (a.w[3] ^ b.w[3])) == 0;
}

__device__ __forceinline__ bool key_less_equal(const Key& a, const Key& b) { return !key_less(b, a); }

// key of entry e < k, reading the second half of e's key only when the first 16 bytes tie
__device__ __forceinline__ bool entry_key_less(const lsm_entry_t* e, const Key& k) {
    const uint4* q = reinterpret_cast<const uint4*>(e);
    const uint4 lo = q[0];
    const uint64_t w0 = __builtin_bswap64(((uint64_t)lo.y << 32) | lo.x);
    const uint64_t w1 = __builtin_bswap64(((uint64_t)lo.w << 32) | lo.z);
    if (w0 != k.w[0]) return w0 < k.w[0];
    if (w1 != k.w[1]) return w1 < k.w[1];
    const uint4 hi = q[1];
    const uint64_t w2 = __builtin_bswap64(((uint64_t)hi.y << 32) | hi.x);
    const uint64_t w3 = __builtin_bswap64(((uint64_t)hi.w << 32) | hi.z);
    if (w2 != k.w[2]) return w2 < k.w[2];
    return w3 < k.w[3];
}

// Number of entries of run[lo, hi) whose key is < k, plus lo.  Global memory.
__device__ __forceinline__ uint64_t lower_bound_run(const lsm_entry_t* run, uint64_t lo, uint64_t hi, const Key& k) {
    while (lo < hi) {
        uint64_t mid = lo + ((hi - lo) >> 1);
        if (entry_key_less(run + mid, k)) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

// Sum / max over the 64 lanes of a wave; every lane must call.
__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v) {
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    for (int off = kWave / 2; off > 0; off >>= 1) {
        uint64_t o = __shfl_xor(v, off, kWave);
        v = o > v ? o : v;
    }
    return v;
}

// 16-byte load through a pointer that is known to be global memory (it went through LDS or a
// table, so the compiler cannot tell): a global instead of a flat load.
__device__ __forceinline__ uint4 load_global_u4(const uint4* p) { typedef uint32_t v4 __attribute__((ext_vector_type(4))); const v4 v = *(const __attribute__((address_space(1))) v4*)p; return make_uint4(v.x, v.y, v.z, v.w); }

// Run descriptors passed to kernels by value.
struct RunTable {
    const lsm_entry_t* ptr[LSM_MAX_RUNS];
    uint64_t n[LSM_MAX_RUNS];
    uint32_t k;
};

}  // namespace lsm
