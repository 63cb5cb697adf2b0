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

// key < k for a key kept as two separate halves (bytes 0..15 at lo, bytes 16..31 at hi); the second
// half is read only when the first 16 bytes tie.
__device__ __forceinline__ bool entry_key_less(const uint4* lo, const uint4* hi, const Key& k) {
    const uint4 a = *lo;
    const uint64_t w0 = __builtin_bswap64(((uint64_t)a.y << 32) | a.x);
    const uint64_t w1 = __builtin_bswap64(((uint64_t)a.w << 32) | a.z);
    if (w0 != k.w[0]) return w0 < k.w[0];
    if (w1 != k.w[1]) return w1 < k.w[1];
    const uint4 b = *hi;
    const uint64_t w2 = __builtin_bswap64(((uint64_t)b.y << 32) | b.x);
    const uint64_t w3 = __builtin_bswap64(((uint64_t)b.w << 32) | b.z);
    if (w2 != k.w[2]) return w2 < k.w[2];
    return w3 < k.w[3];
}

// Three-way compare of a record's key with k (-1, 0, +1) given the record's first 16 key bytes;
// the second half is read only when those tie.
template <typename E>
__device__ __forceinline__ int entry_key_cmp(const E* e, const uint4 lo, const Key& k) {
    const uint64_t w0 = __builtin_bswap64(((uint64_t)lo.y << 32) | lo.x);
    const uint64_t w1 = __builtin_bswap64(((uint64_t)lo.w << 32) | lo.z);
    if (w0 != k.w[0]) return w0 < k.w[0] ? -1 : 1;
    if (w1 != k.w[1]) return w1 < k.w[1] ? -1 : 1;
    const uint4 hi = reinterpret_cast<const uint4*>(e)[1];
    const uint64_t w2 = __builtin_bswap64(((uint64_t)hi.y << 32) | hi.x);
    const uint64_t w3 = __builtin_bswap64(((uint64_t)hi.w << 32) | hi.z);
    if (w2 != k.w[2]) return w2 < k.w[2] ? -1 : 1;
    if (w3 != k.w[3]) return w3 < k.w[3] ? -1 : 1;
    return 0;
}

// The probe position of a search step in [lo, hi), lo < hi: the index with the most trailing zero
// bits.  Positions then form one fixed search tree over the whole array whatever range a search
// starts from, so searches for nearby keys - and repeated searches in a shrinking range - read the
// same few records (the ancestors of the answer) instead of a fresh set of midpoints each time.
__device__ __forceinline__ uint64_t tree_mid(uint64_t lo, uint64_t hi) {
    const uint64_t last = hi - 1, diff = lo ^ last;
    if (diff == 0) return lo;
    const int top = 63 - __builtin_clzll(diff);  // highest bit in which lo and last differ: set in last, clear in lo
    return last & ~((1ull << top) - 1);
}

// Number of records of run[lo, hi) whose key is < k, plus lo (global memory), by bisection along
// the fixed tree.  eq tells whether the record at the result lies inside
// [lo, hi) and has exactly the key k.
template <typename E>
__device__ __forceinline__ uint64_t lower_bound_eq(const E* run, uint64_t lo, uint64_t hi, const Key& k, bool& eq,
                                                   const bool fresh = true) {
    if (fresh) eq = false;  // always describes the record at the current hi
    while (lo < hi) {
        const uint64_t mid = tree_mid(lo, hi);
        const int c = entry_key_cmp(run + mid, *reinterpret_cast<const uint4*>(run + mid), k);
        if (c < 0) lo = mid + 1;
        else hi = mid, eq = c == 0;
    }
    return lo;
}

// The same result by four-way steps at the quartiles of the range (three records read together per
// step): half the dependent round trips for half as many reads again.  For arrays that stay in cache,
// where the round trips are what costs.
template <typename E>
__device__ __forceinline__ uint64_t lower_bound_eq4(const E* run, uint64_t lo, uint64_t hi, const Key& k, bool& eq) {
    eq = false;  // always describes the record at the current hi
    while (hi - lo >= 3) {
        const uint64_t w = hi - lo;
        const uint64_t m1 = lo + (w >> 2), m2 = lo + (w >> 1), m3 = lo + ((3 * w) >> 2);  // lo <= m1 < m2 < m3 < hi
        const uint4 a1 = *reinterpret_cast<const uint4*>(run + m1);
        const uint4 a2 = *reinterpret_cast<const uint4*>(run + m2);
        const uint4 a3 = *reinterpret_cast<const uint4*>(run + m3);
        const int c1 = entry_key_cmp(run + m1, a1, k), c2 = entry_key_cmp(run + m2, a2, k), c3 = entry_key_cmp(run + m3, a3, k);
        if (c3 < 0) {
            lo = m3 + 1;
        } else if (c2 < 0) {
            lo = m2 + 1, hi = m3, eq = c3 == 0;
        } else if (c1 < 0) {
            lo = m1 + 1, hi = m2, eq = c2 == 0;
        } else {
            hi = m1, eq = c1 == 0;
        }
    }
    return lower_bound_eq(run, lo, hi, k, eq, false);  // at most two records left; eq carries over
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

// Bloom filter addressing: the block of a key and the six bits it sets or tests there, as four 32-bit masks.
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ull;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBull;
    x ^= x >> 31;
    return x;
}
// the hash h of a key (its top half picks the block) and the six bits as four 32-bit masks
// h of a key, and the six bits (as a 128-bit mask) that h selects inside its block
__device__ __forceinline__ uint64_t bloom_key_hash(const Key& k) {
    uint64_t h = 0x5EED251116138ull;
    for (int i = 0; i < 4; i++) h = mix64(h ^ k.w[i]);
    return h;
}
__device__ __forceinline__ uint4 bloom_mask(uint64_t h) {
    const uint64_t g = mix64(h ^ 0x9E3779B97F4A7C15ull);
    uint32_t m[4] = {0, 0, 0, 0};
#pragma unroll
    for (int j = 0; j < 6; j++) {
        const uint32_t b = (uint32_t)(g >> (7 * j)) & 127;
#pragma unroll
        for (int w = 0; w < 4; w++) m[w] |= (b >> 5) == (uint32_t)w ? 1u << (b & 31) : 0u;
    }
    return make_uint4(m[0], m[1], m[2], m[3]);
}
__device__ __forceinline__ uint64_t bloom_hash(const Key& k, uint4& mask) {
    const uint64_t h = bloom_key_hash(k);
    mask = bloom_mask(h);
    return h;
}
__device__ __forceinline__ uint32_t bloom_block(uint64_t h, uint32_t n_blocks) { return (uint32_t)(((h >> 32) * (uint64_t)n_blocks) >> 32); }
__device__ __forceinline__ bool bloom_excludes(const uint4 w, const uint4 mask) {
    return (((w.x & mask.x) ^ mask.x) | ((w.y & mask.y) ^ mask.y) | ((w.z & mask.z) ^ mask.z) | ((w.w & mask.w) ^ mask.w)) != 0;
}

// Hash index of a run: 64-byte buckets of kIndexSlots slots.  Bytes 0..15: the slots' 16-bit tag fields (low 15 bits
// = tag; bit 15 of the first field = more keys fall into the bucket than it has slots); bytes 16..47: the slots' 32-bit
// positions, all ones = empty slot; bytes 48..63: zero.
constexpr uint32_t kIndexSlots = 8;
constexpr uint32_t kIndexNoEntry = 0xFFFFFFFFu;
constexpr uint32_t kIndexTagMask = 0x7FFFu;
__host__ __device__ inline uint64_t index_buckets(uint64_t n) { return n ? (n + 3) / 4 : 1; }

// Run descriptors passed to kernels by value.
struct RunTable {
    const lsm_entry_t* ptr[LSM_MAX_RUNS];
    uint64_t n[LSM_MAX_RUNS];  // run lengths; upper bounds when n_dev is given
    const uint64_t* n_dev;     // optional: the run lengths in device memory (written by an earlier kernel of the stream)
    uint32_t k;
};
__device__ __forceinline__ uint64_t run_len(const RunTable& rt, uint32_t j) { return rt.n_dev ? rt.n_dev[j] : rt.n[j]; }

// Compaction of runs whose exact lengths are only known on the device (n_upper[j] >= n_dev[j]; launch sizes come from
// the upper bounds, surplus tiles stay empty).  Used inside the library; arguments are checked by the caller.
// Needs a workspace of lsm_compact_workspace_bytes(n_upper, k) bytes.
int compact_device_lengths(const lsm_entry_t* const* ptr, const uint64_t* n_upper, const uint64_t* n_dev, uint32_t k, uint32_t flags,
                           const lsm_out_t* out, void* workspace, size_t workspace_bytes, hipStream_t stream);

}  // namespace lsm
