// lsm_driver_*: the host driver of one tree.  Level bookkeeping of section 2.2 (a flushed run enters level 1; a level
// that holds more than K runs is merged; a merged run larger than M * T^level moves down), the controller of section
// 3.3 (operation counts over a sliding window, a new (T, K) search when the mix has moved by more than a threshold)
// and the lazy transition of appendix C (a level takes the current T and K when a run next arrives at it).  Nothing
// here touches entries: merging, fence indices, filters, hash indices, lookups and the cost model are the library's
// own entry points.  Merges, flushes and lookups are enqueued on the caller's stream; the lookup structures of a run
// that has come to rest (fence index, filter, hash index) are built on a second stream of the driver's own, beside the
// next compaction: a small merge and the filter of the run before it each keep the GPU busy for some 20 us on a few
// compute units, and nothing but a lookup has to wait for the filter.
//
// Device memory of the runs the driver creates comes from a pool that keeps every block for reuse (hipMalloc and
// hipFree cost more than a small compaction, and hipFree waits for the device).  A block that is given back may still
// be read by work already enqueued on the caller's stream; that is safe because its next user's work is enqueued later
// on the same stream.  Memory that work on the second stream may still touch is given back only after that stream has
// been waited for (finish_builds).
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <deque>
#include <map>
#include <new>
#include <unordered_map>
#include <vector>

#include "lsm_index.h"

namespace {

class DevicePool {
public:
    void* take(size_t bytes) {
        const size_t c = size_class(bytes);
        std::vector<void*>& idle = idle_[c];
        if (!idle.empty()) {
            void* p = idle.back();
            idle.pop_back();
            return p;
        }
        void* p = nullptr;
        if (hipMalloc(&p, c) != hipSuccess) return nullptr;
        size_of_[p] = c;
        return p;
    }
    void give(const void* p) {
        if (p == nullptr) return;
        auto it = size_of_.find(const_cast<void*>(p));
        if (it != size_of_.end()) idle_[it->second].push_back(it->first);
    }
    void free_all() {  // the caller has waited for the stream
        for (auto& kv : size_of_) (void)hipFree(kv.first);
        size_of_.clear();
        idle_.clear();
    }

private:
    // four classes per power of two from 256 bytes up: at most a quarter of a block is unused
    static size_t size_class(size_t bytes) {
        if (bytes > (size_t(1) << 60)) return bytes;  // no such allocation succeeds; keeps the loop below finite
        for (size_t s = 256;; s *= 2)
            for (size_t j = 0; j < 4; j++)
                if (s / 4 * (4 + j) >= bytes) return s / 4 * (4 + j);
    }
    std::map<size_t, std::vector<void*>> idle_;
    std::unordered_map<void*, size_t> size_of_;
};

struct Run {
    const lsm_entry_t* entries = nullptr;
    uint64_t n = 0;
    bool owned = false;      // entries came from the pool
    bool transient = false;  // entries belong to the caller of a flush: copied if the run comes to rest
    uint8_t* fences = nullptr;
    void* bloom = nullptr;
    uint64_t n_blocks = 0;
    void* index = nullptr;
    uint64_t n_buckets = 0;
};

struct Level {
    std::vector<Run> runs;  // newest first
    uint32_t T, K;
};

struct Batch {
    uint64_t writes, hits, empties;
    double blocks;
};

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

}  // namespace

struct lsm_driver {
    lsm_driver_config_t cfg;
    hipStream_t stream = nullptr;  // the caller's
    hipStream_t side = nullptr;    // builds of lookup structures
    hipEvent_t ordered = nullptr;  // makes `side` wait for what `stream` has been given so far
    bool builds_pending = false;
    std::vector<void*> build_scratch;  // temporaries of builds in flight
    double p = 1.0;
    uint32_t T = 0, K = 0;  // what the controller asks for now
    std::vector<Level> levels;
    std::vector<lsm_driver_event_t> log;
    std::deque<Batch> window;
    Batch sum{0, 0, 0, 0.0};
    bool searched = false;
    double last_mix[4] = {0, 0, 0, 0};
    DevicePool pool;
    void* workspace = nullptr;
    size_t workspace_bytes = 0;
    uint64_t* n_host = nullptr;  // pinned: the kernels write a compaction's count here
    uint32_t* hit_host = nullptr;  // pinned copy of a probe batch's hit_len
    size_t hit_host_count = 0;
    uint64_t* counts_host = nullptr;  // pinned: the counts of a batch of compactions (lsm_driver_flush_many)
    size_t counts_host_count = 0;
    void* batch_workspace = nullptr;
    size_t batch_workspace_bytes = 0;

    void record(uint32_t kind, uint32_t level, uint32_t a, uint32_t b, uint64_t n_in, uint64_t n_out) {
        lsm_driver_event_t e;
        std::memset(&e, 0, sizeof(e));
        e.kind = kind, e.level = level, e.a = a, e.b = b, e.n_in = n_in, e.n_out = n_out;
        log.push_back(e);
    }

    void drop(Run& r) {
        if (r.owned) pool.give(r.entries);
        pool.give(r.fences);
        pool.give(r.bloom);
        pool.give(r.index);
        r = Run();
    }

    void ensure_level(uint32_t level) {  // 0-based
        while (levels.size() <= level) levels.push_back(Level{{}, T, K});
    }

    uint64_t total_entries() const {
        uint64_t n = 0;
        for (const Level& lv : levels)
            for (const Run& r : lv.runs) n += r.n;
        return n;
    }

    // M * T^(level + 1), saturating
    uint64_t capacity(uint32_t level) const {
        unsigned __int128 c = cfg.buffer_entries;
        for (uint32_t i = 0; i <= level; i++) {
            c *= levels[level].T;
            if (c > UINT64_MAX) return UINT64_MAX;
        }
        return (uint64_t)c;
    }

    int wait() { return hipStreamSynchronize(stream) == hipSuccess ? LSM_OK : LSM_ERR_HIP; }

    // What the driver needs of the GPU runtime is created by the first call that works on runs, so that the controller
    // (note_writes, note_reads, the log) can be used, and tested, on its own.
    int gpu_ready() {
        if (n_host != nullptr) return LSM_OK;
        if (hipStreamCreateWithFlags(&side, hipStreamNonBlocking) != hipSuccess) return LSM_ERR_HIP;
        if (hipEventCreateWithFlags(&ordered, hipEventDisableTiming) != hipSuccess) return LSM_ERR_HIP;
        return hipHostMalloc(reinterpret_cast<void**>(&n_host), sizeof(uint64_t), hipHostMallocDefault) == hipSuccess ? LSM_OK : LSM_ERR_HIP;
    }

    // Waits for the builds on the second stream.  Needed before a lookup uses the structures, and before any memory the
    // builds read or write goes back to the pool.
    int finish_builds() {
        if (!builds_pending) return LSM_OK;
        builds_pending = false;
        const bool ok = hipStreamSynchronize(side) == hipSuccess;
        for (void* p : build_scratch) pool.give(p);
        build_scratch.clear();
        return ok ? LSM_OK : LSM_ERR_HIP;
    }

    // Filter and hash index of a run that has come to rest; the keys are hashed once for both.  Second stream.
    int build_lookup(Run& r) {
        hipStream_t stream = side;
        auto scratch = [this](size_t bytes) {
            void* p = pool.take(bytes);
            if (p != nullptr) build_scratch.push_back(p);
            return p;
        };
        const bool indexed = cfg.hash_index_from != 0 && r.n >= cfg.hash_index_from && r.n <= (1ull << 27);
        const lsm_run_t run{r.entries, r.n};
        uint64_t* hashes = nullptr;
        int rc = LSM_OK;
        if (indexed) {
            hashes = static_cast<uint64_t*>(scratch(r.n * 8));
            if (hashes == nullptr) return LSM_ERR_HIP;
            rc = lsm_hash_keys(&run, hashes, stream);
        }
        if (rc == LSM_OK && cfg.bloom_bits != 0 && r.bloom == nullptr) {
            r.n_blocks = lsm_bloom_blocks(r.n, cfg.bloom_bits);
            if (r.n_blocks != 0) {
                r.bloom = pool.take(r.n_blocks * 16);
                if (r.bloom == nullptr) rc = LSM_ERR_HIP;
                // a long run: the filter is built from the hashes, sorted by block range (no atomic traffic on the filter)
                const size_t ws_bytes = (hashes != nullptr || r.n >= (1ull << 20)) ? lsm_bloom_workspace_bytes(r.n, r.n_blocks) : 0;
                if (rc == LSM_OK && ws_bytes != 0) {
                    if (hashes == nullptr) {
                        hashes = static_cast<uint64_t*>(scratch(r.n * 8));
                        rc = hashes == nullptr ? (int)LSM_ERR_HIP : lsm_hash_keys(&run, hashes, stream);
                    }
                    void* ws = rc == LSM_OK ? scratch(ws_bytes) : nullptr;
                    if (rc == LSM_OK) rc = ws == nullptr ? (int)LSM_ERR_HIP : lsm_build_bloom_hashed(hashes, r.n, r.bloom, r.n_blocks, ws, ws_bytes, stream);
                } else if (rc == LSM_OK) {
                    rc = lsm_build_bloom(&run, r.bloom, r.n_blocks, stream);
                }
            }
        }
        if (rc == LSM_OK && indexed) {
            r.n_buckets = lsm_hash_index_buckets(r.n);
            const size_t ws_bytes = lsm_hash_index_workspace_bytes(r.n);
            r.index = pool.take(r.n_buckets * 64);
            void* ws = scratch(ws_bytes);
            rc = (r.index == nullptr || ws == nullptr) ? (int)LSM_ERR_HIP : lsm_build_hash_index(hashes, r.n, r.index, ws, ws_bytes, stream);
        }
        return rc;
    }

    // A run that comes to rest in a level gets whatever lookup structure it still lacks.  (Runs that are merged away at
    // once - a flushed run arriving at a full level, a run moved down onto another - never get any.)
    // The entries of a merged run are complete (its count has been waited for, and with it the caller's stream); those of
    // a flushed or loaded run are whatever the caller's stream has been given so far, so the second stream is made to
    // wait for that.
    int settle(Run& r) {
        if (r.n == 0) return LSM_OK;
        const bool from_caller = r.transient || !r.owned;
        if (r.transient) {
            void* copy = pool.take(r.n * sizeof(lsm_entry_t));
            if (copy == nullptr) return LSM_ERR_HIP;
            if (hipMemcpyAsync(copy, r.entries, r.n * sizeof(lsm_entry_t), hipMemcpyDeviceToDevice, stream) != hipSuccess) return LSM_ERR_HIP;
            r.entries = static_cast<const lsm_entry_t*>(copy);
            r.owned = true, r.transient = false;
        }
        if (from_caller && (hipEventRecord(ordered, stream) != hipSuccess || hipStreamWaitEvent(side, ordered, 0) != hipSuccess)) return LSM_ERR_HIP;
        builds_pending = true;
        if (r.fences == nullptr) {
            r.fences = static_cast<uint8_t*>(pool.take(ceil_div(r.n, cfg.fence_stride) * LSM_KEY_BYTES));
            if (r.fences == nullptr) return LSM_ERR_HIP;
            const lsm_run_t run{r.entries, r.n};
            const int rc = lsm_build_fences(&run, cfg.fence_stride, r.fences, side);
            if (rc != LSM_OK) return rc;
        }
        const bool wants_index = cfg.hash_index_from != 0 && r.n >= cfg.hash_index_from && r.n <= (1ull << 27);
        if (r.index == nullptr && (r.bloom == nullptr || wants_index)) return build_lookup(r);  // the filter may be there already (batch)
        return LSM_OK;
    }

    // All runs of a level into one; the fence index of the output is written in the same pass.  Waits for the count
    // (the kernels store it to pinned host memory).  Watching that word from the host instead of synchronising the
    // stream was measured and is no faster: the store becomes visible when the kernel ends.
    int compact(const std::vector<Run>& in, uint32_t flags, uint32_t level, Run* merged) {
        if (in.size() > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
        lsm_run_t runs[LSM_MAX_RUNS];
        uint64_t lens[LSM_MAX_RUNS];
        uint64_t total = 0;
        for (size_t j = 0; j < in.size(); j++) {
            runs[j] = lsm_run_t{in[j].entries, in[j].n};
            lens[j] = in[j].n;
            total += in[j].n;
        }
        const uint32_t k = (uint32_t)in.size();
        const size_t need = lsm_compact_workspace_bytes(lens, k);
        if (need > workspace_bytes) {
            pool.give(workspace);
            workspace_bytes = 2 * need;
            workspace = pool.take(workspace_bytes);
            if (workspace == nullptr) {
                workspace_bytes = 0;
                return LSM_ERR_HIP;
            }
        }
        const uint64_t room = total > 0 ? total : 1;
        lsm_entry_t* entries = static_cast<lsm_entry_t*>(pool.take(room * sizeof(lsm_entry_t)));
        uint8_t* fences = static_cast<uint8_t*>(pool.take(ceil_div(room, cfg.fence_stride) * LSM_KEY_BYTES));
        if (entries == nullptr || fences == nullptr) return LSM_ERR_HIP;
        const lsm_out_t out{entries, room, n_host, fences, cfg.fence_stride, nullptr};
        int rc = lsm_compact(runs, k, flags, &out, workspace, workspace_bytes, stream);
        if (rc == LSM_OK) rc = wait();
        if (rc == LSM_OK && *n_host > room) rc = LSM_ERR_INTERNAL;  // the device-side failure mark, or nonsense
        if (rc != LSM_OK) {
            pool.give(entries);
            pool.give(fences);
            return rc;
        }
        *merged = Run();
        merged->n = *n_host;
        if (cfg.observer != nullptr) cfg.observer(cfg.observer_ctx, level + 1, entries, merged->n);
        if (merged->n == 0) {
            pool.give(entries);
            pool.give(fences);
        } else {
            merged->entries = entries, merged->owned = true, merged->fences = fences;
        }
        return LSM_OK;
    }

    // A run arrives at a level (0-based).  The cascade this starts is cut into steps, so that a caller who drives several
    // trees can run the compactions of their current steps as one batch: arrive_begin places the run and either
    // settles it or leaves a compaction to be done in `due`; arrive_merged takes that compaction's output and either
    // places it, or moves it down (arrive_begin at the next level, which may leave the next compaction in `due`).
    struct Due {
        bool active = false;
        uint32_t level = 0, flags = 0;
        uint64_t n_in = 0;
    } due;

    int arrive_begin(uint32_t level, const Run& moving) {
        ensure_level(level);
        Level& lv = levels[level];
        if (lv.T != T || lv.K != K) record(LSM_EV_ADOPT, level + 1, T, K, 0, 0);
        lv.T = T, lv.K = K;  // lazy transition: the level takes the current parameters when data flows into it
        lv.runs.insert(lv.runs.begin(), moving);
        if (lv.runs.size() <= lv.K) return settle(lv.runs[0]);
        bool deeper_empty = true;
        for (size_t i = level + 1; i < levels.size(); i++) deeper_empty = deeper_empty && levels[i].runs.empty();
        due.active = true, due.level = level, due.flags = deeper_empty ? (uint32_t)LSM_BOTTOMMOST : 0u, due.n_in = 0;
        for (const Run& r : lv.runs) due.n_in += r.n;
        return LSM_OK;
    }

    int arrive_merged(const Run& merged) {
        const uint32_t level = due.level;
        Level& lv = levels[level];
        due.active = false;
        record(LSM_EV_COMPACT, level + 1, (uint32_t)lv.runs.size(), due.flags, due.n_in, merged.n);
        const int built = finish_builds();  // a run that is merged away may still be read by the build of its own filter
        if (built != LSM_OK) return built;
        for (Run& r : lv.runs) drop(r);
        lv.runs.clear();
        if (merged.n > capacity(level)) {
            record(LSM_EV_MOVE, level + 1, level + 2, 0, 0, merged.n);
            return arrive_begin(level + 1, merged);
        }
        if (merged.n > 0) {
            lv.runs.push_back(merged);
            return settle(lv.runs[0]);
        }
        return LSM_OK;
    }

    // The compaction that is due, on its own (one lsm_compact).
    int compact_due() {
        Run merged;
        const int rc = compact(levels[due.level].runs, due.flags, due.level, &merged);
        return rc != LSM_OK ? rc : arrive_merged(merged);
    }

    // The whole cascade of one arrival, one compaction after the other.
    int arrive(uint32_t level, const Run& moving) {
        int rc = arrive_begin(level, moving);
        while (rc == LSM_OK && due.active) rc = compact_due();
        return rc;
    }

    // One batch of operation counts enters the window; the (T, K) search is re-run when the mix has moved.
    int count(uint64_t writes, uint64_t hits, uint64_t empties, double blocks) {
        window.push_back(Batch{writes, hits, empties, blocks});
        sum.writes += writes, sum.hits += hits, sum.empties += empties, sum.blocks += blocks;
        // slide: drop the oldest batches while the rest still covers window_ops operations
        while (window.size() > 1) {
            const Batch& f = window.front();
            if (sum.writes + sum.hits + sum.empties - (f.writes + f.hits + f.empties) < cfg.window_ops) break;
            sum.writes -= f.writes, sum.hits -= f.hits, sum.empties -= f.empties, sum.blocks -= f.blocks;
            window.pop_front();
        }
        const uint64_t total = sum.writes + sum.hits + sum.empties;
        if (total < cfg.window_ops) return LSM_OK;  // the window is not full yet
        const double mix[4] = {(double)sum.writes / (double)total, (double)sum.hits / (double)total / 2, (double)sum.hits / (double)total / 2,
                               (double)sum.empties / (double)total};  // w, s, r, z
        const double d = sum.hits ? sum.blocks / (double)sum.hits : 0.0;
        if (searched) {
            double moved = 0.0;
            for (int i = 0; i < 4; i++) moved += mix[i] > last_mix[i] ? mix[i] - last_mix[i] : last_mix[i] - mix[i];
            if (moved <= cfg.shift_threshold) return LSM_OK;
        }
        std::memcpy(last_mix, mix, sizeof(mix));
        searched = true;
        const uint64_t n = total_entries();
        const lsm_policy_input_t in{mix[0], mix[1], mix[2], mix[3], n > 0 ? n : 1, cfg.buffer_entries, cfg.page_entries, p, d};
        uint32_t best_T = 0, best_K = 0;
        const int rc = lsm_policy_choose(&in, cfg.t_min, cfg.t_max, &best_T, &best_K);
        if (rc != LSM_OK) return rc;
        lsm_driver_event_t e;
        std::memset(&e, 0, sizeof(e));
        e.kind = LSM_EV_POLICY, e.a = best_T, e.b = best_K, e.d = d;
        std::memcpy(e.mix, mix, sizeof(mix));
        log.push_back(e);
        T = best_T, K = best_K;
        return LSM_OK;
    }

    uint32_t tree(lsm_tree_run_t* out, uint32_t capacity) const {
        uint32_t n = 0;
        for (size_t l = 0; l < levels.size(); l++)
            for (const Run& r : levels[l].runs) {
                if (n < capacity) {
                    lsm_tree_run_t t;
                    std::memset(&t, 0, sizeof(t));
                    t.run = lsm_run_t{r.entries, r.n};
                    t.fence = lsm_fence_t{r.fences, r.fences ? ceil_div(r.n, cfg.fence_stride) : 0, cfg.fence_stride};
                    t.bloom = lsm_bloom_t{r.bloom, r.bloom ? r.n_blocks : 0};
                    t.level = (uint32_t)l + 1;
                    t.index = lsm_hash_index_t{r.index, r.index ? r.n_buckets : 0};
                    out[n] = t;
                }
                n++;
            }
        return n;
    }
};

extern "C" int lsm_driver_create(const lsm_driver_config_t* config, void* stream, lsm_driver_t** driver_out) {
    if (config == nullptr || driver_out == nullptr) return LSM_ERR_NULL;
    *driver_out = nullptr;
    if (config->buffer_entries == 0 || config->size_ratio < 2 || config->runs_per_level == 0 || config->window_ops == 0 ||
        config->t_min < 2 || config->t_max < config->t_min || !(config->page_entries > 0) || config->fence_stride == 0)
        return LSM_ERR_BAD_ARG;
    lsm_driver* d = new (std::nothrow) lsm_driver();
    if (d == nullptr) return LSM_ERR_HIP;
    d->cfg = *config;
    d->stream = static_cast<hipStream_t>(stream);
    d->p = config->filter_fpr < 0 ? lsm_policy_filter_fpr(config->bloom_bits) : config->filter_fpr;
    d->T = config->size_ratio, d->K = config->runs_per_level;
    *driver_out = d;
    return LSM_OK;
}

extern "C" void lsm_driver_destroy(lsm_driver_t* d) {
    if (d == nullptr) return;
    if (d->n_host != nullptr || d->side != nullptr) (void)hipStreamSynchronize(d->stream);  // else no GPU call was ever made
    if (d->side != nullptr) (void)hipStreamSynchronize(d->side);
    d->pool.free_all();
    if (d->side != nullptr) (void)hipStreamDestroy(d->side);
    if (d->ordered != nullptr) (void)hipEventDestroy(d->ordered);
    if (d->n_host != nullptr) (void)hipHostFree(d->n_host);
    if (d->hit_host != nullptr) (void)hipHostFree(d->hit_host);
    if (d->counts_host != nullptr) (void)hipHostFree(d->counts_host);
    delete d;
}

extern "C" int lsm_driver_load_run(lsm_driver_t* d, uint32_t level, const lsm_entry_t* entries, uint64_t n) try {
    if (d == nullptr || (n > 0 && entries == nullptr)) return LSM_ERR_NULL;
    if (level == 0 || level > 64 || (reinterpret_cast<uintptr_t>(entries) & 63) != 0) return LSM_ERR_BAD_ARG;
    const int ready = d->gpu_ready();
    if (ready != LSM_OK) return ready;
    d->ensure_level(level - 1);
    Run r;
    r.entries = entries, r.n = n;
    std::vector<Run>& runs = d->levels[level - 1].runs;
    runs.push_back(r);
    return d->settle(runs.back());
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" int lsm_driver_note_writes(lsm_driver_t* d, uint64_t n_ops) try {
    if (d == nullptr) return LSM_ERR_NULL;
    return d->count(n_ops, 0, 0, 0.0);
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" int lsm_driver_note_reads(lsm_driver_t* d, uint64_t successful, uint64_t empty, uint64_t blocks) try {
    if (d == nullptr) return LSM_ERR_NULL;
    if (successful + empty > UINT32_MAX) return LSM_ERR_BAD_ARG;
    d->record(LSM_EV_PROBE, 0, (uint32_t)(successful + empty), (uint32_t)successful, 0, blocks);
    return d->count(0, successful, empty, (double)blocks);
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" int lsm_driver_flush(lsm_driver_t* d, const lsm_entry_t* run, uint64_t n) try {
    if (d == nullptr || (n > 0 && run == nullptr)) return LSM_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(run) & 63) != 0) return LSM_ERR_BAD_ARG;
    const int ready = d->gpu_ready();
    if (ready != LSM_OK) return ready;
    Run r;
    if (n > 0) r.entries = run, r.n = n, r.transient = true;
    return d->arrive(0, r);
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" int lsm_driver_flush_unsorted(lsm_driver_t* d, const lsm_entry_t* buffer, uint64_t n) try {
    if (d == nullptr || (n > 0 && buffer == nullptr)) return LSM_ERR_NULL;
    if (n > LSM_MAX_BUFFER) return LSM_ERR_BAD_ARG;
    const int ready = d->gpu_ready();
    if (ready != LSM_OK) return ready;
    const uint64_t room = n > 0 ? n : 1;
    const size_t ws_bytes = lsm_flush_workspace_bytes(n);
    lsm_entry_t* sorted = static_cast<lsm_entry_t*>(d->pool.take(room * sizeof(lsm_entry_t)));
    void* ws = d->pool.take(ws_bytes > 0 ? ws_bytes : 4);
    uint64_t* n_dev = static_cast<uint64_t*>(d->pool.take(sizeof(uint64_t)));  // the kernels count with atomics: device memory
    int rc = (sorted == nullptr || ws == nullptr || n_dev == nullptr) ? (int)LSM_ERR_HIP : (int)LSM_OK;
    if (rc == LSM_OK) {
        const lsm_out_t out{sorted, room, n_dev, nullptr, 0, nullptr};
        rc = lsm_flush_buffer(buffer, n, &out, ws, ws_bytes > 0 ? ws_bytes : 4, d->stream);
    }
    if (rc == LSM_OK && hipMemcpyAsync(d->n_host, n_dev, sizeof(uint64_t), hipMemcpyDeviceToHost, d->stream) != hipSuccess) rc = LSM_ERR_HIP;
    if (rc == LSM_OK) rc = d->wait();
    d->pool.give(ws);
    d->pool.give(n_dev);
    if (rc == LSM_OK && *d->n_host > room) rc = LSM_ERR_INTERNAL;
    if (rc != LSM_OK) {
        d->pool.give(sorted);
        return rc;
    }
    Run r;
    r.entries = sorted, r.n = *d->n_host, r.owned = true;
    return d->arrive(0, r);
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

// Jobs of at least this many input entries are merged on their own: lsm_compact_batch takes jobs below 2,048 tiles.
static constexpr uint64_t kBatchJobEntries = 1ull << 21;

extern "C" int lsm_driver_flush_many(lsm_driver_t* const* drivers, const lsm_entry_t* const* runs, const uint64_t* n, uint32_t count) try {
    if (count == 0) return LSM_OK;
    if (drivers == nullptr || runs == nullptr || n == nullptr) return LSM_ERR_NULL;
    for (uint32_t i = 0; i < count; i++) {
        if (drivers[i] == nullptr || (n[i] > 0 && runs[i] == nullptr)) return LSM_ERR_NULL;
        if (drivers[i]->stream != drivers[0]->stream || (reinterpret_cast<uintptr_t>(runs[i]) & 63) != 0) return LSM_ERR_BAD_ARG;
        for (uint32_t j = 0; j < i; j++)
            if (drivers[j] == drivers[i]) return LSM_ERR_BAD_ARG;
    }
    lsm_driver_t* const first = drivers[0];
    for (uint32_t i = 0; i < count; i++) {
        const int ready = drivers[i]->gpu_ready();
        if (ready != LSM_OK) return ready;
    }
    if (count > first->counts_host_count) {
        if (first->counts_host != nullptr) (void)hipHostFree(first->counts_host);
        first->counts_host = nullptr, first->counts_host_count = 0;
        if (hipHostMalloc(reinterpret_cast<void**>(&first->counts_host), (size_t)count * sizeof(uint64_t), hipHostMallocDefault) != hipSuccess)
            return LSM_ERR_HIP;
        first->counts_host_count = count;
    }
    for (uint32_t i = 0; i < count; i++) {
        if (runs[i] == nullptr) continue;  // nothing to flush for this tree
        Run r;
        if (n[i] > 0) r.entries = runs[i], r.n = n[i], r.transient = true;
        const int rc = drivers[i]->arrive_begin(0, r);
        if (rc != LSM_OK) return rc;
    }
    std::vector<lsm_driver_t*> active;
    std::vector<std::vector<lsm_run_t>> inputs;
    std::vector<lsm_compact_job_t> jobs;
    std::vector<Run> merged;
    std::vector<lsm_run_t> filtered;
    std::vector<void*> filters;
    std::vector<uint64_t> filter_blocks;
    for (;;) {
        // the compactions that are due now: the long ones on their own, the others as one batch
        active.clear();
        for (uint32_t i = 0; i < count; i++) {
            lsm_driver_t* d = drivers[i];
            while (d->due.active && d->due.n_in >= kBatchJobEntries) {
                const int rc = d->compact_due();
                if (rc != LSM_OK) return rc;
            }
            if (d->due.active) active.push_back(d);
        }
        if (active.empty()) return LSM_OK;
        const uint32_t n_jobs = (uint32_t)active.size();
        inputs.assign(n_jobs, {});
        jobs.assign(n_jobs, lsm_compact_job_t{});
        merged.assign(n_jobs, Run());
        int rc = LSM_OK;
        for (uint32_t j = 0; j < n_jobs && rc == LSM_OK; j++) {
            lsm_driver_t* d = active[j];
            const std::vector<Run>& in = d->levels[d->due.level].runs;
            if (in.size() > LSM_MAX_RUNS) rc = LSM_ERR_BAD_ARG;
            for (const Run& r : in) inputs[j].push_back(lsm_run_t{r.entries, r.n});
            const uint64_t room = d->due.n_in > 0 ? d->due.n_in : 1;
            lsm_entry_t* entries = static_cast<lsm_entry_t*>(d->pool.take(room * sizeof(lsm_entry_t)));
            uint8_t* fences = static_cast<uint8_t*>(d->pool.take(ceil_div(room, d->cfg.fence_stride) * LSM_KEY_BYTES));
            if (entries == nullptr || fences == nullptr) rc = LSM_ERR_HIP;
            merged[j].entries = entries, merged[j].owned = true, merged[j].fences = fences;  // given back through drop() on failure
            jobs[j].runs = inputs[j].data(), jobs[j].n_runs = (uint32_t)inputs[j].size(), jobs[j].flags = d->due.flags;
            jobs[j].out = lsm_out_t{entries, room, first->counts_host + j, fences, d->cfg.fence_stride, nullptr};
        }
        const size_t need = rc == LSM_OK ? lsm_compact_batch_workspace_bytes(jobs.data(), n_jobs) : 0;
        if (rc == LSM_OK && need == 0) rc = LSM_ERR_BAD_ARG;
        if (rc == LSM_OK && need > first->batch_workspace_bytes) {
            first->pool.give(first->batch_workspace);
            first->batch_workspace_bytes = 2 * need;
            first->batch_workspace = first->pool.take(first->batch_workspace_bytes);
            if (first->batch_workspace == nullptr) first->batch_workspace_bytes = 0, rc = LSM_ERR_HIP;
        }
        if (rc == LSM_OK) rc = lsm_compact_batch(jobs.data(), n_jobs, first->batch_workspace, first->batch_workspace_bytes, first->stream);
        if (rc == LSM_OK) rc = first->wait();
        for (uint32_t j = 0; j < n_jobs && rc == LSM_OK; j++)
            if (first->counts_host[j] > jobs[j].out.capacity) rc = LSM_ERR_INTERNAL;  // the device-side failure mark, or nonsense
        if (rc != LSM_OK) {
            for (uint32_t j = 0; j < n_jobs; j++) active[j]->drop(merged[j]);
            return rc;
        }
        // the filters of all outputs in one call
        filtered.clear(), filters.clear(), filter_blocks.clear();
        for (uint32_t j = 0; j < n_jobs; j++) {
            lsm_driver_t* d = active[j];
            merged[j].n = first->counts_host[j];
            if (d->cfg.observer != nullptr) d->cfg.observer(d->cfg.observer_ctx, d->due.level + 1, merged[j].entries, merged[j].n);
            if (merged[j].n == 0) {
                d->drop(merged[j]);
                continue;
            }
            const uint64_t n_blocks = d->cfg.bloom_bits != 0 ? lsm_bloom_blocks(merged[j].n, d->cfg.bloom_bits) : 0;
            if (n_blocks == 0) continue;
            merged[j].bloom = d->pool.take(n_blocks * 16);
            merged[j].n_blocks = n_blocks;
            if (merged[j].bloom == nullptr) rc = LSM_ERR_HIP;
            filtered.push_back(lsm_run_t{merged[j].entries, merged[j].n});
            filters.push_back(merged[j].bloom);
            filter_blocks.push_back(n_blocks);
        }
        if (rc == LSM_OK && !filtered.empty())
            rc = lsm_build_bloom_batch(filtered.data(), filters.data(), filter_blocks.data(), (uint32_t)filtered.size(), first->stream);
        for (uint32_t j = 0; j < n_jobs; j++) {
            if (rc != LSM_OK) {
                active[j]->drop(merged[j]);
                continue;
            }
            rc = active[j]->arrive_merged(merged[j]);
        }
        if (rc != LSM_OK) return rc;
    }
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" int lsm_driver_probe(lsm_driver_t* d, const lsm_queries_t* queries, const lsm_hits_t* out_hits) try {
    if (d == nullptr || queries == nullptr || out_hits == nullptr) return LSM_ERR_NULL;
    lsm_tree_run_t runs[LSM_MAX_RUNS];
    const uint32_t n_runs = d->tree(runs, LSM_MAX_RUNS);
    if (n_runs > LSM_MAX_RUNS) return LSM_ERR_BAD_ARG;
    for (uint32_t i = 0; i < n_runs; i++) runs[i].level = i;
    const lsm_tree_t tree{runs, n_runs};
    int rc = d->gpu_ready();
    if (rc == LSM_OK) rc = d->finish_builds();
    if (rc == LSM_OK) rc = lsm_probe(queries, &tree, out_hits, d->stream);
    if (rc != LSM_OK) return rc;
    const uint32_t n_req = queries->n_req;
    if (n_req > d->hit_host_count) {
        if (d->hit_host != nullptr) (void)hipHostFree(d->hit_host);
        d->hit_host = nullptr, d->hit_host_count = 0;
        if (hipHostMalloc(reinterpret_cast<void**>(&d->hit_host), (size_t)n_req * sizeof(uint32_t), hipHostMallocDefault) != hipSuccess) return LSM_ERR_HIP;
        d->hit_host_count = n_req;
    }
    if (n_req > 0 && hipMemcpyAsync(d->hit_host, out_hits->hit_len, (size_t)n_req * sizeof(uint32_t), hipMemcpyDeviceToHost, d->stream) != hipSuccess)
        return LSM_ERR_HIP;
    rc = d->wait();
    if (rc != LSM_OK) return rc;
    uint64_t hits = 0, blocks = 0;
    for (uint32_t i = 0; i < n_req; i++) {
        hits += d->hit_host[i] > 0;
        blocks += d->hit_host[i];
    }
    d->record(LSM_EV_PROBE, 0, n_req, (uint32_t)hits, 0, blocks);
    return d->count(0, hits, n_req - hits, (double)blocks);
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" uint32_t lsm_driver_levels(const lsm_driver_t* d) { return d ? (uint32_t)d->levels.size() : 0; }

extern "C" int lsm_driver_level(const lsm_driver_t* d, uint32_t level, uint32_t* T, uint32_t* K, uint32_t* n_runs) {
    if (d == nullptr) return LSM_ERR_NULL;
    if (level == 0 || level > d->levels.size()) return LSM_ERR_BAD_ARG;
    const Level& lv = d->levels[level - 1];
    if (T) *T = lv.T;
    if (K) *K = lv.K;
    if (n_runs) *n_runs = (uint32_t)lv.runs.size();
    return LSM_OK;
}

extern "C" int lsm_driver_tree(lsm_driver_t* d, lsm_tree_run_t* runs_out, uint32_t capacity, uint32_t* n_runs) try {
    if (d == nullptr || n_runs == nullptr || (capacity > 0 && runs_out == nullptr)) return LSM_ERR_NULL;
    *n_runs = d->tree(runs_out, capacity);
    return d->finish_builds();
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}

extern "C" int lsm_driver_target(const lsm_driver_t* d, uint32_t* T, uint32_t* K) {
    if (d == nullptr) return LSM_ERR_NULL;
    if (T) *T = d->T;
    if (K) *K = d->K;
    return LSM_OK;
}

extern "C" uint64_t lsm_driver_log(const lsm_driver_t* d, uint64_t first, lsm_driver_event_t* out, uint64_t capacity) {
    if (d == nullptr) return 0;
    const uint64_t n = d->log.size();
    for (uint64_t i = first; out != nullptr && i < n && i - first < capacity; i++) out[i - first] = d->log[i];
    return n;
}

extern "C" int lsm_driver_read(lsm_driver_t* d, const void* device_src, void* dst, size_t bytes) try {
    if (d == nullptr || (bytes > 0 && (device_src == nullptr || dst == nullptr))) return LSM_ERR_NULL;
    int rc = d->gpu_ready();
    if (rc == LSM_OK) rc = d->finish_builds();
    if (rc != LSM_OK) return rc;
    if (bytes > 0 && hipMemcpyAsync(dst, device_src, bytes, hipMemcpyDefault, d->stream) != hipSuccess) return LSM_ERR_HIP;
    return d->wait();
} catch (...) {  // host memory ran out: nothing may be thrown through the C ABI
    return LSM_ERR_INTERNAL;
}
