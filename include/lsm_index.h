/*
 * lsm_index.h -- C ABI of the GPU key index of a key-value-separated LSM-tree.
 *
 * The index stores one 64-byte record per 16-token block of a cached token prefix: a
 * 32-byte prefix-preserving key, a sequence number, a put/tombstone flag and a pointer
 * (file id + offset, length) into separate append-only tensor files (arXiv 2511.16138,
 * section 3.1 "disk index layer" / "tensor-log layer", section 3.2).  This library runs the
 * data-parallel part of that index on one AMD MI355X (gfx950):
 *
 *   lsm_compact       merge sorted runs into one run (section 2.2, compaction); lsm_compact_remap also rewrites
 *                     value pointers for merged tensor files (section 3.4); lsm_compact_batch runs many small
 *                     compactions in one launch; lsm_compact_static allocates nothing
 *   lsm_flush_buffer  the write buffer as a sorted run (section 2.2)
 *   lsm_build_fences  fence-pointer index of a run (section 2.2 names fence pointers)
 *   lsm_build_bloom   Bloom filter of a run (section 2.2 names Bloom filters; appendix B uses them in probes);
 *                     lsm_hash_keys + lsm_build_bloom_hashed build the same filter of a long run from the keys'
 *                     hashes, which lsm_compact can write for its output in its own pass
 *   lsm_build_hash_index  hash index of a run: a lookup finds or rules out a key without the fence search
 *   lsm_probe         batched longest-cached-prefix lookup over a tree (appendix B, "Probe";
 *                     section 2.2, "Point Lookups"); lsm_probe_length gives the length alone by a
 *                     search over the prefix length
 *   lsm_range_scan    the live content of many key ranges (section 2.2, "Range Lookups"; appendix B get_batch);
 *                     lsm_range_bounds: where one key range lies in every run
 *   lsm_policy_*      the adaptive controller's cost model (section 2.2 costs, section 3.3)
 *   lsm_driver_*      the host driver of one tree: levels, the sliding-window controller and the lazy transition of
 *                     (T, K) (section 3.3, appendix C), sequencing the calls above
 *
 * Conventions
 *   - Pointers marked DEVICE are HIP device memory on the current device; pointers marked
 *     HOST are ordinary host memory read during the call only.  Apart from lsm_driver_* (a driver
 *     object owns the runs it creates), the library never allocates or frees device memory and
 *     keeps no state between calls; the caller owns every buffer.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream).
 *     Calls return as soon as the work is enqueued unless stated otherwise; outputs are
 *     valid once the stream has been synchronised.
 *   - Every function returns 0 (LSM_OK) or a negative lsm_status; nothing throws or aborts.
 *     Argument errors are detected on the host before anything is launched, so a call
 *     that fails with one of them has written nothing.  (LSM_ERR_UNSORTED / LSM_ERR_BAD_ENTRY / LSM_ERR_INTERNAL
 *     are found on the device: the workspace, and for LSM_ERR_INTERNAL the output, have been written by then.)
 *   - Keys are ordered as 32-byte big-endian byte strings (memcmp order).  All other fields
 *     are little-endian.  There is no floating point on the device.
 */
#ifndef LSM_INDEX_H
#define LSM_INDEX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* One index record.  64 bytes, natural alignment, no packing pragma needed. */
typedef struct {
    uint8_t  key[32]; /* prefix-preserving key; order = memcmp(a.key, b.key, 32)           */
    uint64_t seqno;   /* larger = newer (unsigned)                                          */
    uint8_t  type;    /* LSM_PUT or LSM_TOMBSTONE                                           */
    uint8_t  pad0[7]; /* carried through verbatim                                           */
    uint64_t vptr;    /* (file_id << 32) | offset in the tensor log; opaque to this library */
    uint32_t vlen;    /* bytes of the tensor block; opaque                                  */
    uint32_t pad1;    /* carried through verbatim                                           */
} lsm_entry_t;

enum { LSM_PUT = 0, LSM_TOMBSTONE = 1 };

/* flags of lsm_compact */
enum {
    LSM_BOTTOMMOST = 1, /* output is the last level: winning tombstones are dropped too   */
    LSM_VALIDATE = 2    /* check inputs (strictly ascending runs, type byte); synchronises */
};

typedef enum {
    LSM_OK = 0,
    LSM_ERR_NULL = -1,      /* a required pointer is NULL                                  */
    LSM_ERR_BAD_ARG = -2,   /* n_runs == 0 or too large, stride == 0, max_blocks too large */
    LSM_ERR_CAPACITY = -3,  /* out->capacity < total number of input entries               */
    LSM_ERR_WORKSPACE = -4, /* workspace missing, misaligned or too small                  */
    LSM_ERR_UNSORTED = -5,  /* LSM_VALIDATE: a run is not strictly ascending by key        */
    LSM_ERR_BAD_ENTRY = -6, /* LSM_VALIDATE: a type byte is neither PUT nor TOMBSTONE      */
    LSM_ERR_HIP = -7,       /* a HIP call failed                                           */
    LSM_ERR_INTERNAL = -8,  /* a device-side consistency check failed (see lsm_compact)    */
    LSM_ERR_STATIC_LIMIT = -9 /* lsm_compact_static: the input needs more scratch than the library's static array holds */
} lsm_status;

enum {
    LSM_MAX_RUNS = 64,          /* runs per lsm_compact call and per lsm_tree_t            */
    LSM_MAX_BLOCKS = 256,       /* block keys per probe request                            */
    LSM_MAX_BUFFER = 262144,    /* entries per lsm_flush_buffer call                       */
    LSM_RANGE_MAX_ENTRIES = 2048, /* entries one range of lsm_range_scan may hold (all versions) */
    LSM_KEY_BYTES = 32,
    LSM_STATIC_SCRATCH_BYTES = 8 << 20, /* scratch held inside the library for lsm_compact_static      */
    LSM_DEFAULT_FENCE_STRIDE = 64 /* one fence per 4 KiB page of entries                   */
};

/* A sorted run: n entries, strictly ascending by key (one version per key per run). */
typedef struct {
    const lsm_entry_t* entries; /* DEVICE, 64-byte aligned */
    uint64_t n;
} lsm_run_t;

/* Destination of a compaction. */
typedef struct {
    lsm_entry_t* entries; /* DEVICE, 64-byte aligned, room for `capacity` entries           */
    uint64_t capacity;    /* must be >= the total number of input entries                   */
    uint64_t* n_out;      /* DEVICE (or host memory the device can write, e.g. pinned), one
                           * uint64: number of entries written                               */
    /* Optional: the fence index of the new run, written in the same pass (what lsm_build_fences
     * would give for it).  fence_keys: DEVICE, 16-byte aligned, room for ceil(capacity / fence_stride)
     * keys of 32 bytes, of which the first ceil(*n_out / fence_stride) are written; NULL = none. */
    uint8_t* fence_keys;
    uint32_t fence_stride; /* > 0 if fence_keys is given */
    /* Optional: key_hashes[i] = the filter hash h (see lsm_bloom_t) of output entry i, written in the same
     * pass, so that the filter of the new run can be built by lsm_build_bloom_hashed without reading the
     * run again.  DEVICE, 8-byte aligned, room for `capacity` values; NULL = none.  Honoured by lsm_compact,
     * lsm_compact_timed, lsm_compact_remap and lsm_compact_static; lsm_flush_buffer and lsm_compact_batch
     * reject a request for it (LSM_ERR_BAD_ARG): their outputs are short. */
    uint64_t* key_hashes;
} lsm_out_t;

/* Fence index of a run: fence i is the key of entry i*stride. */
typedef struct {
    const uint8_t* keys; /* DEVICE, n x 32 bytes, n = ceil(run.n / stride); may be NULL if run.n == 0 */
    uint64_t n;
    uint32_t stride;
} lsm_fence_t;

/*
 * Bloom filter of a run (section 2.2: lookups go through Bloom filters and fence pointers; the
 * false-positive rate is the p of the lookup costs).  The paper does not fix a filter format; this one is a
 * blocked filter with 128-bit blocks, so that a lookup reads one 16-byte word:
 *   k_i   = key bytes 8i .. 8i+7 read as a big-endian 64-bit number, i = 0..3
 *   mix(x): x ^= x >> 30; x *= 0xBF58476D1CE4E5B9; x ^= x >> 27; x *= 0x94D049BB133111EB; x ^= x >> 31
 *           (64-bit arithmetic; the output function of the splitmix64 generator)
 *   h = 0x5EED251116138; for i = 0..3: h = mix(h ^ k_i);   g = mix(h ^ 0x9E3779B97F4A7C15)
 *   block = ((h >> 32) * n_blocks) >> 32;   bit_j = (g >> (7 j)) & 127 for j = 0..5
 * A key is in the filter when the six bits are set in its block; bit b of a block is bit (b & 31) of the
 * block's little-endian 32-bit word b >> 5.  No false negatives; about 0.2 % false positives at 16 bits per key (lsm_policy_filter_fpr).
 */
typedef struct {
    const void* blocks; /* DEVICE, n_blocks x 16 bytes, 16-byte aligned; NULL = the run has no filter */
    uint64_t n_blocks;  /* < 2^32 */
} lsm_bloom_t;

/*
 * Hash index of a run (optional; built by lsm_build_hash_index).  Section 2.2 has a point lookup consult a run's
 * Bloom filter and then its fence pointers; with the run in device memory the fence search is a dozen dependent
 * reads.  The hash index answers both questions - can the key be in this run, and where - from one 64-byte line:
 *   n_buckets = lsm_hash_index_buckets(n) = max(1, ceil(n / 4)) buckets of 64 bytes, eight slots each
 *   a key with filter hash h (the h of lsm_bloom_t) belongs to bucket ((h >> 32) * n_buckets) >> 32; tag = h & 0x7FFF
 *   bytes  0..15  the slots' tag fields, 16 bits each (little-endian): low 15 bits = tag of the key in the slot
 *                 (0 for an empty slot); bit 15 is set in the first field only, and only when more than eight
 *                 keys of the run fall into the bucket ("crowded": it then holds eight of them)
 *   bytes 16..47  the slots' positions in the run, 32 bits each; 0xFFFFFFFF = empty slot
 *   bytes 48..63  zero
 * A key whose tag is in no slot of its uncrowded bucket is not in the run, so a lookup reads the 16 tag bytes where
 * it would read a filter block, and the index does what the filter does; a lookup that does not find its key in a
 * crowded bucket searches the fence index instead.  Which eight keys a crowded bucket keeps and the order of the
 * slots inside a bucket are not defined; lookups give the same answers for every table of this form.  Runs of at
 * most 2^27 entries.
 */
typedef struct {
    const void* buckets; /* DEVICE, 64-byte aligned, n_buckets x 64 bytes; NULL = none */
    uint64_t n_buckets;  /* = lsm_hash_index_buckets(run.n) if buckets is given */
} lsm_hash_index_t;

typedef struct {
    lsm_run_t run;
    lsm_fence_t fence;
    lsm_bloom_t bloom; /* optional: lsm_probe skips the run for keys the filter excludes */
    uint32_t level;    /* informational */
    lsm_hash_index_t index; /* optional: lsm_probe finds (or rules out) a key in the run without the fence search */
} lsm_tree_run_t;

/* A tree = its runs ordered NEWEST -> OLDEST (shallow level first; within a level, the most
 * recently written run first).  Precondition (LSM invariant): if a key is present in several
 * runs, the run that comes earlier in this array holds the larger seqno. */
typedef struct {
    const lsm_tree_run_t* runs; /* HOST array */
    uint32_t n_runs;            /* <= LSM_MAX_RUNS */
} lsm_tree_t;

/* A batch of probe requests; request r asks for n_blocks[r] consecutive block keys. */
typedef struct {
    const uint8_t* keys;      /* DEVICE, n_req x max_blocks x 32 bytes, row-major           */
    const uint32_t* n_blocks; /* DEVICE, n_req values, each <= max_blocks                   */
    uint32_t n_req;
    uint32_t max_blocks;      /* row pitch in keys; <= LSM_MAX_BLOCKS                       */
} lsm_queries_t;

typedef struct {
    uint64_t vptr;
    uint32_t vlen;
    uint32_t run_idx; /* index into tree.runs of the run that held the newest version       */
} lsm_hit_t;

typedef struct {
    uint32_t* hit_len; /* DEVICE, n_req                                                     */
    lsm_hit_t* hits;   /* DEVICE, n_req x max_blocks; all-zero at and beyond hit_len[r]     */
} lsm_hits_t;

/*
 * lsm_compact -- merge n_runs sorted runs into one sorted run (section 2.2: data of smaller
 * levels is merged into larger ones, sorted order is kept, obsolete entries are removed).
 *
 * Result: for every distinct key of the inputs, the version with the largest seqno (equal
 * seqnos: the one from the lowest run index; runs[0] is the newest run) -- except that a
 * winning TOMBSTONE is dropped when LSM_BOTTOMMOST is set.  Survivors are written to
 * out->entries in strictly ascending key order as byte-for-byte copies of the winning 64
 * input bytes, and their count is stored to *out->n_out.  The inputs are not modified and
 * must not overlap the output.
 *
 * runs        HOST array of n_runs descriptors (1 <= n_runs <= LSM_MAX_RUNS); empty runs allowed.
 * workspace   DEVICE scratch of at least lsm_compact_workspace_bytes(...) bytes, 256-byte
 *             aligned; contents on entry are irrelevant.
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG, LSM_ERR_CAPACITY, LSM_ERR_WORKSPACE, LSM_ERR_HIP.
 * With LSM_VALIDATE the call synchronises the stream and additionally returns
 * LSM_ERR_UNSORTED / LSM_ERR_BAD_ENTRY (checked before merging; nothing is written then) or
 * LSM_ERR_INTERNAL.  Without it, inputs that violate the precondition give an unspecified
 * (but in-bounds) result.
 * The output offset of a tile comes from the counts of the tiles before it; a tile waits for them, and tile numbers
 * are workgroup numbers, so the wait relies on workgroups being started in ascending order (which holds on this
 * hardware also when several kernels share the GPU, but is not a documented guarantee).  The wait is bounded: if it
 * ever ends without the counts, the remaining tiles write nothing, *out->n_out is set to UINT64_MAX instead of a
 * count, and the output is incomplete - every caller that does not use LSM_VALIDATE should check for that value when
 * it reads the count.  Two compactions may run at the same time on two streams if each has its own workspace.
 */
int lsm_compact(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                size_t workspace_bytes, void* stream);

/*
 * lsm_compact_timed -- lsm_compact with optional timing hooks: the three HIP events (hipEvent_t
 * handles owned by the caller, any of them may be NULL) are recorded on `stream` before the
 * partition kernel, before the tile-merge kernel and after it, so a caller can measure the
 * kernels of one call with hipEventElapsedTime.  ev == NULL is exactly lsm_compact.
 */
typedef struct {
    void* before_partition;
    void* before_merge;
    void* after_merge;
} lsm_compact_events_t;

int lsm_compact_timed(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                      size_t workspace_bytes, void* stream, const lsm_compact_events_t* ev);

/*
 * lsm_compact_remap -- lsm_compact that also rewrites the value pointers of the entries it writes (section 3.4,
 * automatic tensor-file merging: tensor files are merged in the background as part of the compaction schedule, and
 * the file id and offset stored in the index entries then have to follow).  A value pointer is (file_id << 32) | offset.  For every
 * surviving PUT whose file_id < n_files:  vptr_out = base[file_id] + offset  (64-bit addition; base[f] is the new
 * (file_id << 32) | offset of old file f's first byte).  Other entries - tombstones, files outside the table -
 * are copied unchanged.  base: DEVICE, n_files x uint64.  remap == NULL or n_files == 0 is exactly lsm_compact.
 * ev may be NULL (see lsm_compact_timed).  Errors as lsm_compact, plus LSM_ERR_NULL for a table without base.
 */
typedef struct {
    const uint64_t* base;
    uint32_t n_files;
} lsm_remap_t;

int lsm_compact_remap(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* workspace,
                      size_t workspace_bytes, void* stream, const lsm_remap_t* remap, const lsm_compact_events_t* ev);

/*
 * lsm_compact_static -- lsm_compact without a workspace argument, for callers that cannot allocate device memory:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The scratch memory is a
 * static device array of LSM_STATIC_SCRATCH_BYTES (8 MiB) inside the library, which every GPU the library runs on
 * holds until the process ends; the call allocates and frees nothing.  The caller still passes inputs and outputs.
 * Limit: inputs with lsm_compact_workspace_bytes(...) > LSM_STATIC_SCRATCH_BYTES (about 4 million entries for 16
 * runs) are rejected with LSM_ERR_STATIC_LIMIT before anything is launched.  LSM_VALIDATE is rejected with
 * LSM_ERR_BAD_ARG (it copies to the host and waits).  All calls on one GPU share that GPU's array: calls that
 * overlap in time on one GPU (two streams, two threads) race and give undefined results; calls that follow each
 * other on one stream are fine, whatever their sizes.  Result and other errors exactly as lsm_compact.
 */
int lsm_compact_static(const lsm_run_t* runs, uint32_t n_runs, uint32_t flags, const lsm_out_t* out, void* stream);

/* Bytes of workspace lsm_compact needs for runs of these lengths (HOST array). 0 on bad arguments.
 * About one byte per input entry (a copy of every 32nd key) plus 24 * n_runs bytes per (2048 - n_runs) entries. */
size_t lsm_compact_workspace_bytes(const uint64_t* run_lens, uint32_t n_runs);

/*
 * lsm_flush_buffer -- the write buffer as a sorted run (section 2.2: writes go to an in-memory buffer that is
 * flushed as a sorted run when it is full).  buffer: DEVICE, 64-byte aligned, n <= LSM_MAX_BUFFER entries in the
 * order they were written, possibly several versions of a key.  Result: ascending by key, one entry per key -
 * the one with the largest seqno, and among equal seqnos the one written last; tombstones are entries like any
 * other.  out as for lsm_compact (capacity >= n; fence_keys optional).  workspace: DEVICE scratch of at least
 * lsm_flush_workspace_bytes(n) bytes, 256-byte aligned (4 * n bytes up to 8,192 entries; beyond that about 70 bytes
 * per entry: room for the sorted segments and for the merge).  Up to 8,192 entries every entry is compared with
 * every other (key compares from LDS); a larger buffer is cut into segments of 4,096 entries in write order, the
 * segments are sorted that way in one launch and then merged by the compaction kernels.  The call does not wait.
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (n > LSM_MAX_BUFFER, misaligned), LSM_ERR_CAPACITY, LSM_ERR_WORKSPACE, LSM_ERR_HIP.
 */
size_t lsm_flush_workspace_bytes(uint64_t n);
int lsm_flush_buffer(const lsm_entry_t* buffer, uint64_t n, const lsm_out_t* out, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * lsm_build_fences -- fence_keys_out[i] = run->entries[i*stride].key for 0 <= i < ceil(n/stride)
 * (fence pointers, section 2.2: one key per page of `stride` entries, used to find the page
 * that may hold a key without reading the run).
 * fence_keys_out: DEVICE, ceil(n/stride) x 32 bytes.  Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (stride == 0).
 */
int lsm_build_fences(const lsm_run_t* run, uint32_t stride, uint8_t* fence_keys_out, void* stream);

/*
 * lsm_build_bloom -- Bloom filter of a run in the format described at lsm_bloom_t.
 * lsm_bloom_blocks(n, bits_per_key) = max(1, ceil(n * bits_per_key / 128)) blocks of 16 bytes (0 if that is
 * 2^32 or more, or bits_per_key is 0).  filter_out: DEVICE, 16-byte aligned, n_blocks x 16 bytes, overwritten
 * (cleared, then every key of the run inserted).  The result does not depend on the order of insertion.
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (n_blocks == 0 or >= 2^32, misaligned pointers), LSM_ERR_HIP.
 */
uint64_t lsm_bloom_blocks(uint64_t n, uint32_t bits_per_key);
int lsm_build_bloom(const lsm_run_t* run, void* filter_out, uint64_t n_blocks, void* stream);

/*
 * lsm_build_bloom_batch -- the filters of n_runs runs in two launches per 64 runs (for the outputs of
 * lsm_compact_batch): filters_out[j] receives the filter of runs[j] with n_blocks[j] blocks, each exactly what
 * lsm_build_bloom gives.  runs, filters_out, n_blocks: HOST arrays of n_runs elements; the pointers inside are DEVICE.
 * Errors as lsm_build_bloom.
 */
int lsm_build_bloom_batch(const lsm_run_t* runs, void* const* filters_out, const uint64_t* n_blocks, uint32_t n_runs, void* stream);

/*
 * lsm_hash_keys, lsm_build_bloom_hashed -- the same filter for a long run, built from the keys' hashes without
 * read-modify-write traffic on the filter (section 2.2 has every new run carry a filter, so the build is part
 * of every compaction's cost).  lsm_hash_keys writes hashes_out[i] = h of entry i's key (the h of lsm_bloom_t;
 * DEVICE, 8-byte aligned, run->n values); lsm_compact can write the same values for its output in its own
 * pass (lsm_out_t.key_hashes).  lsm_build_bloom_hashed sorts the n hashes into ranges of 4,096 filter blocks
 * inside the workspace, builds each range in on-chip memory and writes it once; filter_out as for
 * lsm_build_bloom and with the same bytes as its result.  The hashes are only read.
 * lsm_bloom_workspace_bytes(n, n_blocks): bytes the build needs (DEVICE, 256-byte aligned, about 8 n), or 0
 * when it does not apply (n >= 2^32, n_blocks == 0 or more than 2^25 blocks: use lsm_build_bloom).
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (as lsm_build_bloom; not applicable), LSM_ERR_WORKSPACE, LSM_ERR_HIP.
 */
size_t lsm_bloom_workspace_bytes(uint64_t n, uint64_t n_blocks);
int lsm_hash_keys(const lsm_run_t* run, uint64_t* hashes_out, void* stream);
int lsm_build_bloom_hashed(const uint64_t* hashes, uint64_t n, void* filter_out, uint64_t n_blocks, void* workspace,
                           size_t workspace_bytes, void* stream);

/*
 * lsm_build_hash_index -- the hash index of a run (see lsm_hash_index_t) from the filter hashes of its keys in
 * run order (hashes[i] belongs to entry i: from lsm_hash_keys, or from lsm_compact's key_hashes).  buckets_out:
 * DEVICE, 64-byte aligned, lsm_hash_index_buckets(n) x 64 bytes, every byte written.  The hashes are sorted by
 * ranges of 4,096 buckets inside the workspace and every range is filled by one workgroup (no atomic traffic
 * on the table).  lsm_hash_index_workspace_bytes(n): DEVICE, 256-byte aligned, about 16 n bytes; 0 when the
 * build does not apply (n > 2^27).
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (misaligned pointers, n too large), LSM_ERR_WORKSPACE, LSM_ERR_HIP.
 */
uint64_t lsm_hash_index_buckets(uint64_t n);
size_t lsm_hash_index_workspace_bytes(uint64_t n);
int lsm_build_hash_index(const uint64_t* hashes, uint64_t n, void* buckets_out, void* workspace, size_t workspace_bytes, void* stream);

/*
 * lsm_probe -- batched longest-cached-prefix lookup (appendix B "Probe": find the longest
 * cached prefix of a request; section 2.2 "Point Lookups": levels are checked in order and
 * the first match is the result).
 *
 * For request r with keys q[0..n): newest(q[j]) is the version of q[j] in the first run of
 * `tree` (newest -> oldest) that contains it; q[j] is live if that version exists and is a PUT.
 * hit_len[r] = number of leading live keys (first-miss semantics: a hole ends the prefix even
 * if later blocks are present).  hits[r][j] = {vptr, vlen, run index} of newest(q[j]) for
 * j < hit_len[r], and 16 zero bytes for hit_len[r] <= j < max_blocks.
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (max_blocks == 0 or > LSM_MAX_BLOCKS, n_runs > LSM_MAX_RUNS,
 * a run with n > 0 whose fence index is missing or has n != ceil(run.n/stride)), LSM_ERR_HIP.
 * n_req == 0 and n_runs == 0 are legal (every request then has hit_len 0).
 */
int lsm_probe(const lsm_queries_t* queries, const lsm_tree_t* tree, const lsm_hits_t* out_hits, void* stream);

/*
 * lsm_probe_length -- only the length of the longest cached prefix, found as appendix B describes "Probe": by a
 * search over the prefix length with point lookups, not by a lookup of every block key.  Valid on PREFIX-CLOSED
 * data: whenever block j of a request is live, blocks 0..j-1 are live too (what leaf-first eviction of cached
 * sequences gives).  hit_len: DEVICE, n_req values; on such data equal to lsm_probe's.  On other data the value is
 * some j with block j-1 live (or j == 0) and block j not live (or j == n_blocks).  About 67 point lookups for a
 * request of 256 blocks, in two dependent rounds.  Errors as lsm_probe.
 */
int lsm_probe_length(const lsm_queries_t* queries, const lsm_tree_t* tree, uint32_t* hit_len, void* stream);

/*
 * lsm_range_bounds -- where a key range starts and ends in every run of a tree: the first step of a range lookup
 * (section 2.2, range lookups; appendix B: get_batch first scans a key range of the index for the keys and the
 * places of their tensors).  lo_key, hi_key: HOST, 32 bytes each.  bounds_out: DEVICE, 2 * n_runs uint64:
 *   bounds_out[2r] = number of entries of run r with key < lo_key, bounds_out[2r+1] = number with key < hi_key.
 * The range's content is then one lsm_compact with LSM_BOTTOMMOST over the slices
 * runs[r].entries[bounds[2r] .. bounds[2r+1]) (newest version of every key in [lo_key, hi_key), live PUTs only).
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG, LSM_ERR_HIP.
 */
int lsm_range_bounds(const lsm_tree_t* tree, const uint8_t* lo_key, const uint8_t* hi_key, uint64_t* bounds_out, void* stream);

/*
 * lsm_range_scan -- the content of many key ranges in one call (appendix B, get_batch: range scans over the index give
 * the keys of the cached blocks under a prefix and the places of their tensors; section 2.2, range lookups).
 * For range i, [lo_keys[i], hi_keys[i]): the entries of the tree whose key lies in the range, newest version of each
 * key, live PUTs only, ascending - what a last-level lsm_compact of the runs cut to the range gives.  They are written
 * to out->entries[i * max_entries ...] (whole 64-byte entries: key, value pointer and length make the read list for
 * the tensor files) and their number to out->counts[i].  One workgroup handles one range: it finds the range in every
 * run and merges the pieces like a tile of a compaction.  A range whose pieces hold more than LSM_RANGE_MAX_ENTRIES
 * entries in all, or whose result has more than max_entries, gets counts[i] = LSM_RANGE_OVERFLOW and nothing
 * meaningful in its slot: use lsm_range_bounds and lsm_compact for it.  lo >= hi is an empty range.
 * lo_keys, hi_keys: DEVICE, n_ranges x 32 bytes, 16-byte aligned.  entries: DEVICE, 64-byte aligned,
 * n_ranges x max_entries entries.  counts: DEVICE, n_ranges.  Fence indices and filters of the tree are not used.
 * Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (max_entries == 0 or > LSM_RANGE_MAX_ENTRIES, misaligned), LSM_ERR_HIP.
 */
typedef struct {
    const uint8_t* lo_keys;
    const uint8_t* hi_keys;
    uint32_t n_ranges;
    uint32_t max_entries; /* slot pitch of the result, in entries */
} lsm_ranges_t;

typedef struct {
    lsm_entry_t* entries;
    uint32_t* counts;
} lsm_range_out_t;

#define LSM_RANGE_OVERFLOW 0xFFFFFFFFu

int lsm_range_scan(const lsm_ranges_t* ranges, const lsm_tree_t* tree, const lsm_range_out_t* out, void* stream);

/*
 * lsm_compact_batch -- many independent small compactions in one call (section 2.2: the flush / compaction cycle of
 * the small upper levels; with several trees or key-range shards their compactions do not depend on each other).
 * Job j merges jobs[j].runs into jobs[j].out exactly as lsm_compact would with jobs[j].flags; all jobs share two
 * kernel launches (one partition, one tile merge), and every job's count goes to its own out.n_out on the device.
 * out.fence_keys works as in lsm_compact.  Restrictions: LSM_VALIDATE is not supported here; a job of 2048 tiles or
 * more (about 4 million entries) is rejected with LSM_ERR_BAD_ARG - use lsm_compact for it.  Inputs and outputs of different jobs must not
 * overlap.  jobs, and the run arrays they point to: HOST, read during the call.  workspace: DEVICE, 256-byte
 * aligned, lsm_compact_batch_workspace_bytes(jobs, n_jobs) bytes (0 on bad arguments); the call copies a table of
 * the jobs into it (built in pinned host memory that the library keeps per calling thread; a call waits for the
 * table copy of the previous call from the same thread, not for its kernels).  Errors as lsm_compact.
 */
typedef struct {
    const lsm_run_t* runs; /* HOST array of n_runs descriptors */
    uint32_t n_runs;
    uint32_t flags;
    lsm_out_t out;
} lsm_compact_job_t;

size_t lsm_compact_batch_workspace_bytes(const lsm_compact_job_t* jobs, uint32_t n_jobs);
int lsm_compact_batch(const lsm_compact_job_t* jobs, uint32_t n_jobs, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Cost model of the adaptive controller (host only, double arithmetic).
 *   L = smallest integer >= 1 with buffer_entries * T^L >= n_entries     (section 2.2: L = log_T(N e / M))
 *   W = T L / (B K)   update;  Z = K L p  empty point lookup;  R = K L p + 1  non-empty point
 *   lookup;  S = K L + d / B  range lookup                                (section 2.2)
 *   cost = w W + s S + r R + z Z                                         (section 3.3)
 * w, s, r, z are the observed shares of writes, range reads, successful point reads and empty
 * probes in the current window.  lsm_policy_choose scans T in [t_min, t_max], K in [1, T-1]
 * (K = 1 leveling ... K = T-1 tiering) and returns the cheapest pair; equal costs go to the
 * smaller K, then the smaller T.  Errors: LSM_ERR_NULL, LSM_ERR_BAD_ARG (t_min < 2, t_max < t_min,
 * buffer_entries == 0, B <= 0).
 */
typedef struct {
    double w, s, r, z;       /* workload mix                                   */
    uint64_t n_entries;      /* N                                              */
    uint64_t buffer_entries; /* M / e                                          */
    double B;                /* entries per page                               */
    double p;                /* Bloom-filter false-positive rate (1 = no filter) */
    double d;                /* entries returned by a range lookup             */
} lsm_policy_input_t;

uint32_t lsm_policy_levels(uint64_t n_entries, uint64_t buffer_entries, uint32_t T);
double lsm_policy_cost(const lsm_policy_input_t* in, uint32_t T, uint32_t K);
int lsm_policy_choose(const lsm_policy_input_t* in, uint32_t t_min, uint32_t t_max, uint32_t* best_T,
                      uint32_t* best_K);

/*
 * lsm_policy_filter_fpr -- the false-positive rate p of the lookup costs (section 2.2) for a run filtered by
 * lsm_build_bloom with `bits_per_key` bits per key: the expectation, over the Poisson number of keys that share a
 * 128-bit block, of the probability that six bits drawn for a foreign key are all set.  0 bits per key = no filter:
 * returns 1.  About 0.0022 at 16 bits per key.
 */
double lsm_policy_filter_fpr(uint32_t bits_per_key);

/*
 * lsm_driver_* -- the host driver of one tree: level bookkeeping (section 2.2: flushed runs enter level 1, a level
 * holds at most K runs and M * T^level entries, full levels are merged and overflowing ones moved down), the
 * adaptive controller (section 3.3: operation counts over a sliding window, a new (T, K) search when the mix has
 * moved by more than a threshold) and the lazy transition (appendix C: a level takes the current T and K when data
 * next flows into it; a smaller K merges the level at that arrival, a larger K leaves it alone).  It sequences the
 * calls above on the caller's stream (the lookup structures of a run that has come to rest are built on a second
 * stream of the driver's own, beside the next compaction; lookups and inspection wait for them) and owns the device
 * memory of the runs it creates (a pool that is given back only by lsm_driver_destroy).  One thread at a time per
 * driver.  Every call returns an lsm_status (LSM_ERR_HIP also when device memory runs out, LSM_ERR_INTERNAL also when
 * host memory does); after an error other than LSM_ERR_NULL / LSM_ERR_BAD_ARG the driver's tree is undefined and it
 * can only be destroyed.
 *
 * Readings where the paper gives no constants: an operation is one inserted sequence (lsm_driver_note_writes) or one
 * probe request; a request that finds no live first block is an empty probe (z), the others count half as range
 * reads (s) and half as point reads (r); d = mean number of blocks a successful request found; N = entries in the
 * tree at the time of the search; the window is the shortest suffix of the reported batches that covers window_ops
 * operations, and no search is made before it is that long; "moved" = L1 distance of (w, s, r, z) to the mix of the
 * last search > shift_threshold.
 */
typedef struct lsm_driver lsm_driver_t;

enum { LSM_EV_ADOPT = 1, LSM_EV_COMPACT = 2, LSM_EV_MOVE = 3, LSM_EV_PROBE = 4, LSM_EV_POLICY = 5 };

/* One record of the driver's log.  Levels are 1-based.
 *   ADOPT    level takes over new parameters:  level, a = T, b = K
 *   COMPACT  all runs of a level merged:       level, a = number of runs, b = flags, n_in, n_out = entries in / out
 *   MOVE     merged run moved down:            level = from, a = to, n_out = its entries
 *   PROBE    one probe batch:                  a = requests, b = requests with hit_len > 0, n_out = sum of hit_len
 *   POLICY   a (T, K) search:                  a = T, b = K, mix = (w, s, r, z), d                                */
typedef struct {
    uint32_t kind, level, a, b;
    uint64_t n_in, n_out;
    double mix[4];
    double d;
} lsm_driver_event_t;

/* Called after every compaction, when its output is complete (the stream has been waited for): entries is DEVICE
 * memory owned by the driver, valid only during the call. */
typedef void (*lsm_driver_observer_t)(void* ctx, uint32_t level, const lsm_entry_t* entries, uint64_t n);

typedef struct {
    uint64_t buffer_entries;  /* M: entries of a full write buffer (> 0)                                 */
    uint32_t size_ratio;      /* T the levels start with (>= 2)                                          */
    uint32_t runs_per_level;  /* K the levels start with (>= 1)                                          */
    uint64_t window_ops;      /* operations the sliding window covers                                    */
    double shift_threshold;   /* L1 distance of the mix that triggers a new search                       */
    uint32_t t_min, t_max;    /* range of T the search may choose from (t_min >= 2)                      */
    double page_entries;      /* B of the cost model                                                     */
    double filter_fpr;        /* p of the cost model; negative = lsm_policy_filter_fpr(bloom_bits)       */
    uint32_t fence_stride;    /* > 0                                                                     */
    uint32_t bloom_bits;      /* bits per key of the runs' filters; 0 = no filters                       */
    uint64_t hash_index_from; /* runs of at least this many entries also get a hash index; 0 = none      */
    lsm_driver_observer_t observer; /* may be NULL */
    void* observer_ctx;
} lsm_driver_config_t;

/* stream: the HIP stream all of the driver's work is enqueued on (NULL = the default stream). */
int lsm_driver_create(const lsm_driver_config_t* config, void* stream, lsm_driver_t** driver_out);
/* Waits for the stream, frees everything the driver allocated. NULL is allowed. */
void lsm_driver_destroy(lsm_driver_t* driver);

/* The starting tree: appends a run as the OLDEST run of `level` (1-based) without merging anything, and builds its
 * fence index, filter and hash index.  entries: DEVICE, borrowed - it must stay valid until the run has been merged
 * away (it no longer appears in lsm_driver_tree) or the driver is destroyed; the driver never frees it. */
int lsm_driver_load_run(lsm_driver_t* driver, uint32_t level, const lsm_entry_t* entries, uint64_t n);

/* n_ops sequences were inserted since the last report (the controller's write count). */
int lsm_driver_note_writes(lsm_driver_t* driver, uint64_t n_ops);

/* Lookups answered elsewhere (the caller's own lsm_probe calls over lsm_driver_tree, say): `successful` requests
 * that found `blocks` blocks in all, and `empty` requests that found nothing; logged and counted like one probe batch.
 * Neither this call nor lsm_driver_note_writes touches the GPU. */
int lsm_driver_note_reads(lsm_driver_t* driver, uint64_t successful, uint64_t empty, uint64_t blocks);

/* A sorted run from the write buffer enters level 1; every compaction and move this triggers is done before the call
 * returns.  run: DEVICE, strictly ascending; it is read only by work that the call enqueues on the driver's stream (a
 * run that comes to rest is copied), so the caller may reuse the memory in stream order afterwards. */
int lsm_driver_flush(lsm_driver_t* driver, const lsm_entry_t* run, uint64_t n);
/* The same for a write buffer as it was filled (any order, repeated keys; n <= LSM_MAX_BUFFER): sorted and reduced to
 * the newest version of every key by lsm_flush_buffer first. */
int lsm_driver_flush_unsorted(lsm_driver_t* driver, const lsm_entry_t* buffer, uint64_t n);

/* One flush for each of `count` independent trees (key-range shards of one index, or one index per tenant), stepped
 * together: the compactions that the trees' cascades need at the same step go to the GPU as one lsm_compact_batch (the
 * fence indices written in the same pass) and the filters of their outputs as one lsm_build_bloom_batch, until every tree
 * is settled; a compaction of 2^21 entries or more is run on its own.  Every tree ends exactly as after its own
 * lsm_driver_flush.  drivers, runs, n: HOST arrays of `count` elements; runs[i] == NULL = tree i has nothing to flush
 * (an empty write buffer, which is still a flush, is a non-NULL runs[i] with n[i] == 0).
 * The drivers must be distinct and share one stream (LSM_ERR_BAD_ARG otherwise). */
int lsm_driver_flush_many(lsm_driver_t* const* drivers, const lsm_entry_t* const* runs, const uint64_t* n, uint32_t count);

/* lsm_probe over the current tree (run_idx of a hit = position in lsm_driver_tree's order); the call waits for the
 * result, counts the batch in the window and may re-run the (T, K) search.  More than LSM_MAX_RUNS runs in the tree:
 * LSM_ERR_BAD_ARG. */
int lsm_driver_probe(lsm_driver_t* driver, const lsm_queries_t* queries, const lsm_hits_t* out_hits);

/* Inspection.  lsm_driver_levels: number of levels.  lsm_driver_level: the parameters level `level` (1-based) runs
 * with and its number of runs.  lsm_driver_tree: the runs newest -> oldest with their lookup structures (`level`
 * field = 1-based level), at most `capacity` of them, *n_runs = how many there are; the call waits until the
 * structures are built, and the DEVICE pointers stay valid until the next flush.  lsm_driver_target: the (T, K) the controller currently asks for.  lsm_driver_log: copies
 * records first .. first + capacity - 1 of the log and returns the total number of records.  lsm_driver_read: waits
 * for the stream and copies `bytes` bytes of driver-owned DEVICE memory to dst (HOST or DEVICE). */
uint32_t lsm_driver_levels(const lsm_driver_t* driver);
int lsm_driver_level(const lsm_driver_t* driver, uint32_t level, uint32_t* T, uint32_t* K, uint32_t* n_runs);
int lsm_driver_tree(lsm_driver_t* driver, lsm_tree_run_t* runs_out, uint32_t capacity, uint32_t* n_runs);
int lsm_driver_target(const lsm_driver_t* driver, uint32_t* T, uint32_t* K);
uint64_t lsm_driver_log(const lsm_driver_t* driver, uint64_t first, lsm_driver_event_t* out, uint64_t capacity);
int lsm_driver_read(lsm_driver_t* driver, const void* device_src, void* dst, size_t bytes);

const char* lsm_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* LSM_INDEX_H */
