// Subgroup-to-tier allocation proportional to path bandwidth (Eq. 1 of the paper) and its online re-estimation
// (Section 3.3).  Host logic only.
#include <math.h>

#include <vector>

#include "mlpo_internal.h"

using namespace mlpo;

namespace {

// Eq. 1 over the tiers listed in `live`, for `m` subgroups: ceilings of the proportional shares, then the surplus is
// taken back one subgroup at a time from the tier that would finish last (largest count / bandwidth; among equals the
// one with the lower bandwidth, then the higher index), so that the paths finish as close together as they can.
void proportional(int64_t m, const std::vector<int>& live, const double* bw, int32_t* count) {
    double total = 0.0;
    for (int i : live) total += bw[i];
    int64_t sum = 0;
    for (int i : live) {
        const double share = (double)m * bw[i] / total;
        int64_t c = (int64_t)ceil(share - 1e-12);
        if (c < 0) c = 0;
        count[i] = (int32_t)c;
        sum += c;
    }
    while (sum > m) {
        int worst = -1;
        for (int i : live) {
            if (count[i] == 0) continue;
            if (worst < 0) {
                worst = i;
                continue;
            }
            const double a = (double)count[i] / bw[i], b = (double)count[worst] / bw[worst];
            if (a > b || (a == b && (bw[i] < bw[worst] || (bw[i] == bw[worst] && i > worst)))) worst = i;
        }
        --count[worst];
        --sum;
    }
}

}  // namespace

extern "C" {

int mlpo_assign_tiers(int32_t n_subgroups, int32_t n_tiers, const double* bandwidth, const int32_t* capacity,
                      int32_t* count, int32_t* tier_of_subgroup) {
    if (n_subgroups < 0 || n_tiers < 1 || n_tiers > 64) return fail(MLPO_EINVAL, "bad subgroup or tier count");
    if (bandwidth == nullptr || count == nullptr) return fail(MLPO_EINVAL, "bandwidth or count is NULL");
    for (int i = 0; i < n_tiers; ++i)
        if (!(isfinite(bandwidth[i]) && bandwidth[i] > 0.0))
            return fail(MLPO_EINVAL, "bandwidth of tier %d must be finite and > 0", i);
    std::vector<int> live;
    for (int i = 0; i < n_tiers; ++i) {
        count[i] = 0;
        live.push_back(i);
    }
    // A tier that cannot hold its proportional share keeps what it can hold; Eq. 1 is applied again to what is left.
    int64_t left = n_subgroups;
    while (left > 0) {
        if (live.empty()) return fail(MLPO_ENOMEM, "the tiers' capacities add up to less than %d subgroups", n_subgroups);
        std::vector<int32_t> trial((size_t)n_tiers, 0);
        proportional(left, live, bandwidth, trial.data());
        bool clamped = false;
        for (size_t q = 0; q < live.size();) {
            const int i = live[q];
            if (capacity != nullptr && capacity[i] >= 0 && trial[(size_t)i] > capacity[i]) {
                count[i] = capacity[i];
                left -= capacity[i];
                live.erase(live.begin() + (long)q);
                clamped = true;
            } else {
                ++q;
            }
        }
        if (!clamped) {
            for (int i : live) count[i] = trial[(size_t)i];
            left = 0;
        }
    }
    if (tier_of_subgroup != nullptr) {
        // Slower tiers take the lower subgroup ids: after an ascending pass the high ids are the ones left on the
        // fast tiers (Section 3.2 "Cache-Friendly Ordering").
        std::vector<int> by_speed;
        for (int i = 0; i < n_tiers; ++i) by_speed.push_back(i);
        for (size_t a = 0; a < by_speed.size(); ++a)
            for (size_t b = a + 1; b < by_speed.size(); ++b)
                if (bandwidth[by_speed[b]] < bandwidth[by_speed[a]] ||
                    (bandwidth[by_speed[b]] == bandwidth[by_speed[a]] && by_speed[b] > by_speed[a])) {
                    const int t = by_speed[a];
                    by_speed[a] = by_speed[b];
                    by_speed[b] = t;
                }
        int32_t next = 0;
        for (int i : by_speed)
            for (int32_t k = 0; k < count[i]; ++k) tier_of_subgroup[next++] = i;
    }
    return MLPO_OK;
}

int mlpo_update_bandwidth(int32_t n_tiers, double* bandwidth, const double* bytes_moved, const double* seconds) {
    if (n_tiers < 1 || bandwidth == nullptr || bytes_moved == nullptr || seconds == nullptr)
        return fail(MLPO_EINVAL, "bad arguments");
    for (int i = 0; i < n_tiers; ++i) {
        if (!(bytes_moved[i] >= 0.0) || !(seconds[i] >= 0.0)) return fail(MLPO_EINVAL, "negative observation for tier %d", i);
        // a tier that moved nothing in the last iteration keeps its estimate
        if (bytes_moved[i] > 0.0 && seconds[i] > 0.0) bandwidth[i] = bytes_moved[i] / seconds[i];
    }
    return MLPO_OK;
}

}  // extern "C"
