/*
 * CPU checker for the LSM key index.  TEST INFRASTRUCTURE ONLY: this file is what the GPU
 * library's results are compared against.  Nothing in the library links, includes or calls
 * it, and it shares no code with the library.  It is written for obviousness, not speed.
 *
 * What it computes (paper: arXiv 2511.16138, "KV Stores Scale Up KV Cache"):
 *   - key order            section 3.1 / 3.2: keys are encoded so that lexicographic order is
 *                          prefix order; here a key is 32 bytes compared as a byte string.
 *   - compaction           section 2.2 ("LSM-Tree Structure"): sorted runs are merged, sorted
 *                          order is kept and obsolete entries are removed.
 *   - point lookup, probe  section 2.2 ("Point Lookups"): every level is checked and the
 *                          matching (newest) entry is the result; appendix B ("Probe"): the
 *                          longest cached prefix of a request.
 *   - fence pointers       section 2.2 names them; fence i is the key of entry i*stride.
 *   - cost model           section 2.2 (update / point / range lookup costs) and section 3.3
 *                          (weighted sum w*W + s*S + r*R + z*Z, minimised over T and K).
 *
 * Every function below has an independent pin in tests/test_oracle_*.py (brute force in
 * Python on tiny inputs, invariants, reductions to sorted()/bisect, closed forms).
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    uint8_t  key[32];
    uint64_t seqno;
    uint8_t  type; /* 0 = PUT, 1 = TOMBSTONE */
    uint8_t  pad0[7];
    uint64_t vptr;
    uint32_t vlen;
    uint32_t pad1;
} entry_t;

typedef struct {
    uint64_t vptr;
    uint32_t vlen;
    uint32_t run_idx;
} hit_t;

enum { FLAG_BOTTOMMOST = 1 };
enum { TYPE_PUT = 0, TYPE_TOMBSTONE = 1 };

/* Key order: byte-string comparison of the 32 key bytes. */
int oracle_key_cmp(const uint8_t* a, const uint8_t* b) { return memcmp(a, b, 32); }

/* ------------------------------------------------------------------------------------
 * Compaction: heap-based k-way merge.
 * The heap holds the current head of every non-exhausted run, smallest first under
 * (key ascending, seqno descending, run index ascending).  Entries therefore leave the
 * heap grouped by key with the newest version of each key first: that one is the winner,
 * the rest of the group is obsolete and is dropped.  A winning tombstone is dropped only
 * when the output is the last level (nothing older can remain below it).
 * runs[0] is the newest run; it only matters as the tie-break for equal seqnos.
 * Returns the number of entries written to out (capacity: the total input count).
 * ------------------------------------------------------------------------------------ */
typedef struct {
    const entry_t* const* runs;
    const uint64_t* pos;
} heap_ctx_t;

static int head_before(const heap_ctx_t* c, uint32_t ra, uint32_t rb) {
    const entry_t* a = &c->runs[ra][c->pos[ra]];
    const entry_t* b = &c->runs[rb][c->pos[rb]];
    int k = memcmp(a->key, b->key, 32);
    if (k != 0) return k < 0;
    if (a->seqno != b->seqno) return a->seqno > b->seqno;
    return ra < rb;
}

static void sift_down(const heap_ctx_t* c, uint32_t* heap, uint32_t n, uint32_t i) {
    for (;;) {
        uint32_t l = 2 * i + 1, r = l + 1, m = i;
        if (l < n && head_before(c, heap[l], heap[m])) m = l;
        if (r < n && head_before(c, heap[r], heap[m])) m = r;
        if (m == i) return;
        uint32_t t = heap[i];
        heap[i] = heap[m];
        heap[m] = t;
        i = m;
    }
}

uint64_t oracle_compact(const entry_t* const* runs, const uint64_t* lens, uint32_t n_runs, uint32_t flags,
                        entry_t* out) {
    uint64_t* pos = (uint64_t*)calloc(n_runs ? n_runs : 1, sizeof(uint64_t));
    uint32_t* heap = (uint32_t*)malloc((n_runs ? n_runs : 1) * sizeof(uint32_t));
    heap_ctx_t ctx = {runs, pos};
    uint32_t hn = 0;
    for (uint32_t r = 0; r < n_runs; r++)
        if (lens[r] > 0) heap[hn++] = r;
    for (uint32_t i = hn / 2; i-- > 0;) sift_down(&ctx, heap, hn, i);

    uint64_t n_out = 0;
    int have_last = 0;
    uint8_t last_key[32];
    while (hn > 0) {
        uint32_t r = heap[0];
        const entry_t* e = &runs[r][pos[r]];
        if (!have_last || memcmp(e->key, last_key, 32) != 0) {
            /* first (= newest) entry of a new key group */
            memcpy(last_key, e->key, 32);
            have_last = 1;
            if (!((flags & FLAG_BOTTOMMOST) && e->type == TYPE_TOMBSTONE)) out[n_out++] = *e;
        }
        pos[r]++;
        if (pos[r] == lens[r]) heap[0] = heap[--hn];
        sift_down(&ctx, heap, hn, 0);
    }
    free(pos);
    free(heap);
    return n_out;
}

/* ------------------------------------------------------------------------------------
 * Probe: linear scan over the request's block keys; for each key every run of the tree is
 * searched (no early exit, no fences) and the version with the largest seqno is taken
 * (ties: lowest run index).  A key is live if that version exists and is a PUT.
 * hit_len = number of leading live keys; hits[j] is filled for j < hit_len and zero after.
 * qkeys: n_req x max_blocks x 32 bytes; hits: n_req x max_blocks.
 * ------------------------------------------------------------------------------------ */
static uint64_t lower_bound(const entry_t* run, uint64_t n, const uint8_t* key) {
    uint64_t lo = 0, hi = n;
    while (lo < hi) {
        uint64_t mid = lo + (hi - lo) / 2;
        if (memcmp(run[mid].key, key, 32) < 0) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

void oracle_probe(const uint8_t* qkeys, const uint32_t* n_blocks, uint32_t n_req, uint32_t max_blocks,
                  const entry_t* const* runs, const uint64_t* lens, uint32_t n_runs, uint32_t* hit_len,
                  hit_t* hits) {
    for (uint32_t q = 0; q < n_req; q++) {
        hit_t* row = hits + (uint64_t)q * max_blocks;
        memset(row, 0, sizeof(hit_t) * max_blocks);
        uint32_t j = 0;
        for (; j < n_blocks[q]; j++) {
            const uint8_t* key = qkeys + ((uint64_t)q * max_blocks + j) * 32;
            const entry_t* best = NULL;
            uint32_t best_run = 0;
            for (uint32_t r = 0; r < n_runs; r++) {
                uint64_t i = lower_bound(runs[r], lens[r], key);
                if (i < lens[r] && memcmp(runs[r][i].key, key, 32) == 0) {
                    if (best == NULL || runs[r][i].seqno > best->seqno) {
                        best = &runs[r][i];
                        best_run = r;
                    }
                }
            }
            if (best == NULL || best->type != TYPE_PUT) break;
            row[j].vptr = best->vptr;
            row[j].vlen = best->vlen;
            row[j].run_idx = best_run;
        }
        hit_len[q] = j;
    }
}

/* Fence index: fence[i] = key of entry i*stride, for 0 <= i < ceil(n/stride). */
void oracle_build_fences(const entry_t* run, uint64_t n, uint32_t stride, uint8_t* fence_keys) {
    uint64_t i = 0;
    for (uint64_t e = 0; e < n; e += stride, i++) memcpy(fence_keys + 32 * i, run[e].key, 32);
}

/* ------------------------------------------------------------------------------------
 * Bloom filter of a run (section 2.2: lookups use Bloom filters and fence pointers).  The
 * paper fixes no format; the one checked here is the library's documented one, written out
 * bit by bit: blocks of 128 bits, six bits per key inside one block.
 *   k_i = key bytes 8i..8i+7 as a big-endian number; mix = output function of splitmix64
 *   h = 0x5EED251116138; h = mix(h ^ k_i) for i = 0..3; g = mix(h ^ 0x9E3779B97F4A7C15)
 *   block = ((h >> 32) * n_blocks) >> 32; bits (g >> 7j) & 127, j = 0..5
 * A filter is stored as bytes: bit b of a block lives in byte b / 8, bit b % 8 (that is the
 * little-endian 32-bit-word layout of the library).
 * ------------------------------------------------------------------------------------ */
static uint64_t splitmix_out(uint64_t x) {
    x ^= x >> 30;
    x *= 0xBF58476D1CE4E5B9ULL;
    x ^= x >> 27;
    x *= 0x94D049BB133111EBULL;
    x ^= x >> 31;
    return x;
}

static void bloom_place(const uint8_t* key, uint64_t n_blocks, uint64_t* block, unsigned bits[6]) {
    uint64_t h = 0x5EED251116138ULL;
    for (int i = 0; i < 4; i++) {
        uint64_t k = 0;
        for (int b = 0; b < 8; b++) k = (k << 8) | key[8 * i + b];
        h = splitmix_out(h ^ k);
    }
    uint64_t g = splitmix_out(h ^ 0x9E3779B97F4A7C15ULL);
    *block = ((h >> 32) * n_blocks) >> 32;
    for (int j = 0; j < 6; j++) bits[j] = (unsigned)((g >> (7 * j)) & 127);
}

uint64_t oracle_bloom_blocks(uint64_t n, uint32_t bits_per_key) {
    if (bits_per_key == 0) return 0;
    unsigned __int128 bits = (unsigned __int128)n * bits_per_key;
    unsigned __int128 blocks = bits == 0 ? 1 : (bits + 127) / 128;
    return blocks >= ((unsigned __int128)1 << 32) ? 0 : (uint64_t)blocks;
}

void oracle_build_bloom(const entry_t* run, uint64_t n, uint8_t* filter, uint64_t n_blocks) {
    memset(filter, 0, 16 * n_blocks);
    for (uint64_t e = 0; e < n; e++) {
        uint64_t block;
        unsigned bits[6];
        bloom_place(run[e].key, n_blocks, &block, bits);
        for (int j = 0; j < 6; j++) filter[16 * block + bits[j] / 8] |= (uint8_t)(1u << (bits[j] % 8));
    }
}

/* 1 if the filter may contain the key, 0 if it certainly does not */
int oracle_bloom_may_contain(const uint8_t* filter, uint64_t n_blocks, const uint8_t* key) {
    uint64_t block;
    unsigned bits[6];
    bloom_place(key, n_blocks, &block, bits);
    for (int j = 0; j < 6; j++)
        if (!(filter[16 * block + bits[j] / 8] & (1u << (bits[j] % 8)))) return 0;
    return 1;
}

/* ------------------------------------------------------------------------------------
 * Hash index of a run (the library's own in-memory index beside the filter and the fence pointers of section 2.2;
 * its format is stated with lsm_hash_index_t in the library's header).  The index is not unique - which eight keys
 * a crowded bucket keeps and the order of the slots are left open - so the checker does not build one: it decides
 * whether a given table is a valid index of a given run.
 *   h(key) as for the filter above; bucket = ((h >> 32) * n_buckets) >> 32; tag = h & 0x7FFF
 *   n_buckets = max(1, ceil(n / 4)); a bucket is 64 bytes with eight slots:
 *   bytes 0..15 tag fields (16 bits each, little-endian; bit 15 of the first = crowded, 0 for an empty slot),
 *   bytes 16..47 positions (32 bits each, all ones = empty), bytes 48..63 zero
 *   more than 8 keys in a bucket: 8 of them and the crowded bit
 * Returns 0 for a valid table, else the number of the rule that is broken.
 * ------------------------------------------------------------------------------------ */
static uint64_t key_hash(const uint8_t* key) {
    uint64_t h = 0x5EED251116138ULL;
    for (int i = 0; i < 4; i++) {
        uint64_t k = 0;
        for (int b = 0; b < 8; b++) k = (k << 8) | key[8 * i + b];
        h = splitmix_out(h ^ k);
    }
    return h;
}

void oracle_key_hashes(const entry_t* run, uint64_t n, uint64_t* out) {
    for (uint64_t e = 0; e < n; e++) out[e] = key_hash(run[e].key);
}

uint64_t oracle_hash_index_buckets(uint64_t n) { return n ? (n + 3) / 4 : 1; }

int oracle_hash_index_check(const entry_t* run, uint64_t n, const uint8_t* table, uint64_t n_buckets) {
    if (n_buckets != oracle_hash_index_buckets(n)) return 1;
    uint32_t* keys_of = calloc(n_buckets, sizeof(uint32_t)); /* how many keys of the run belong to each bucket */
    uint8_t* listed = calloc(n ? n : 1, 1);                  /* entry e appears in the table */
    int rc = 0;
    for (uint64_t e = 0; e < n; e++) keys_of[((key_hash(run[e].key) >> 32) * n_buckets) >> 32]++;
    for (uint64_t b = 0; b < n_buckets && rc == 0; b++) {
        const uint8_t* bucket = table + 64 * b;
        uint32_t held = 0;
        const int crowded = (bucket[1] & 0x80) != 0;
        for (int k = 0; k < 8 && rc == 0; k++) {
            const uint32_t field = (uint32_t)bucket[2 * k] | (uint32_t)bucket[2 * k + 1] << 8;
            uint32_t pos = 0;
            for (int i = 3; i >= 0; i--) pos = pos << 8 | bucket[16 + 4 * k + i];
            if (k > 0 && (field & 0x8000)) rc = 8; /* bit 15 belongs to the first field only */
            else if (pos == 0xFFFFFFFFu) {
                if (field & 0x7FFF) rc = 9; /* an empty slot has tag 0 */
            } else if (pos >= n) rc = 2;     /* points outside the run */
            else {
                const uint64_t h = key_hash(run[pos].key);
                if ((((h >> 32) * n_buckets) >> 32) != b || (h & 0x7FFF) != (field & 0x7FFF)) rc = 3; /* wrong bucket or wrong tag */
                else if (listed[pos]) rc = 4;                                                           /* listed twice */
                else listed[pos] = 1, held++;
            }
        }
        for (int i = 48; i < 64 && rc == 0; i++)
            if (bucket[i]) rc = 10; /* the rest of the bucket is zero */
        if (rc) break;
        if (keys_of[b] <= 8) {
            if (crowded) rc = 5;                 /* marked crowded without need */
            else if (held != keys_of[b]) rc = 6; /* a key is missing: a lookup would not find it */
        } else if (!crowded || held != 8) rc = 7;
    }
    free(keys_of);
    free(listed);
    return rc;
}

/* ------------------------------------------------------------------------------------
 * Cost model of the adaptive controller.
 *   levels   L = smallest integer >= 1 with M * T^L >= N   (L = log_T(N*e/M), in entries)
 *   update   W = T*L / (B*K)
 *   empty point lookup      Z = K*L*p
 *   non-empty point lookup  R = K*L*p + 1
 *   range lookup            S = K*L + d/B
 *   cost     = w*W + s*S + r*R + z*Z
 * oracle_policy_choose scans T in [t_min, t_max] and K in [1, T-1] and keeps the smallest
 * cost; equal costs go to the smaller K, then to the smaller T.
 * ------------------------------------------------------------------------------------ */
uint32_t oracle_levels(uint64_t n_entries, uint64_t buffer_entries, uint32_t T) {
    uint32_t L = 1;
    long double cap = (long double)buffer_entries * T;
    while (cap < (long double)n_entries) {
        cap *= T;
        L++;
    }
    return L;
}

double oracle_cost(double w, double s, double r, double z, uint64_t n_entries, uint64_t buffer_entries,
                   uint32_t T, uint32_t K, double B, double p, double d) {
    double L = (double)oracle_levels(n_entries, buffer_entries, T);
    double W = (double)T * L / (B * (double)K);
    double Z = (double)K * L * p;
    double R = (double)K * L * p + 1.0;
    double S = (double)K * L + d / B;
    return w * W + s * S + r * R + z * Z;
}

void oracle_policy_choose(double w, double s, double r, double z, uint64_t n_entries, uint64_t buffer_entries,
                          uint32_t t_min, uint32_t t_max, double B, double p, double d, uint32_t* best_T,
                          uint32_t* best_K) {
    double best = 0.0;
    int have = 0;
    for (uint32_t T = t_min; T <= t_max; T++) {
        for (uint32_t K = 1; K + 1 <= T; K++) {
            double c = oracle_cost(w, s, r, z, n_entries, buffer_entries, T, K, B, p, d);
            if (!have || c < best || (c == best && (K < *best_K || (K == *best_K && T < *best_T)))) {
                best = c;
                have = 1;
                *best_T = T;
                *best_K = K;
            }
        }
    }
}
