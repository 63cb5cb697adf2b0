// Cost model of the adaptive controller (paper section 2.2 operation costs, section 3.3
// weighted total) and the status strings.  Host code only.
#include <math.h>
#include <stdint.h>

#include "lsm_index.h"

extern "C" uint32_t lsm_policy_levels(uint64_t n_entries, uint64_t buffer_entries, uint32_t T) {
    if (buffer_entries == 0 || T < 2) return 0;
    // smallest L >= 1 with buffer_entries * T^L >= n_entries, in exact integer arithmetic
    unsigned __int128 cap = (unsigned __int128)buffer_entries * T;
    uint32_t L = 1;
    while (cap < (unsigned __int128)n_entries) {
        cap *= T;
        L++;
    }
    return L;
}

extern "C" double lsm_policy_cost(const lsm_policy_input_t* in, uint32_t T, uint32_t K) {
    if (in == nullptr || K == 0 || T < 2 || in->buffer_entries == 0 || !(in->B > 0.0)) return -1.0;
    const double L = (double)lsm_policy_levels(in->n_entries, in->buffer_entries, T);
    const double W = (double)T * L / (in->B * (double)K);
    const double Z = (double)K * L * in->p;
    const double R = (double)K * L * in->p + 1.0;
    const double S = (double)K * L + in->d / in->B;
    return in->w * W + in->s * S + in->r * R + in->z * Z;
}

extern "C" int lsm_policy_choose(const lsm_policy_input_t* in, uint32_t t_min, uint32_t t_max, uint32_t* best_T,
                                 uint32_t* best_K) {
    if (in == nullptr || best_T == nullptr || best_K == nullptr) return LSM_ERR_NULL;
    if (t_min < 2 || t_max < t_min || in->buffer_entries == 0 || !(in->B > 0.0)) return LSM_ERR_BAD_ARG;
    bool have = false;
    double best = 0.0;
    for (uint32_t T = t_min; T <= t_max; T++) {
        for (uint32_t K = 1; K < T; K++) {
            const double c = lsm_policy_cost(in, T, K);
            const bool better = !have || c < best || (c == best && (K < *best_K || (K == *best_K && T < *best_T)));
            if (better) {
                have = true;
                best = c;
                *best_T = T;
                *best_K = K;
            }
        }
    }
    return LSM_OK;
}

// p of the lookup costs for the blocked filter of lsm_build_bloom: a block of 128 bits receives a Poisson number of
// keys (mean 128 / bits_per_key), each key sets six bits drawn with repetition, and a key that was never inserted
// passes when its own six bits are all set.
extern "C" double lsm_policy_filter_fpr(uint32_t bits_per_key) {
    if (bits_per_key == 0) return 1.0;
    const double mean = 128.0 / (double)bits_per_key;
    double weight = exp(-mean), p = 0.0;  // Poisson weight of a block with no key: such a block passes nothing
    const int last = (int)(mean + 12.0 * sqrt(mean) + 50.0);
    for (int keys = 1; keys <= last; keys++) {
        weight *= mean / (double)keys;
        const double bit_set = 1.0 - pow(1.0 - 1.0 / 128.0, 6.0 * (double)keys);
        p += weight * pow(bit_set, 6.0);
    }
    return p;
}

extern "C" const char* lsm_strerror(int code) {
    switch (code) {
        case LSM_OK: return "ok";
        case LSM_ERR_NULL: return "a required pointer is NULL";
        case LSM_ERR_BAD_ARG: return "bad argument";
        case LSM_ERR_CAPACITY: return "output capacity smaller than the total input size";
        case LSM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LSM_ERR_UNSORTED: return "an input run is not strictly ascending by key";
        case LSM_ERR_BAD_ENTRY: return "an input entry has an invalid type byte";
        case LSM_ERR_HIP: return "a HIP call failed";
        case LSM_ERR_INTERNAL: return "device-side consistency check failed";
        case LSM_ERR_STATIC_LIMIT: return "input too large for the library's static scratch (use lsm_compact with a workspace)";
        default: return "unknown status";
    }
}
