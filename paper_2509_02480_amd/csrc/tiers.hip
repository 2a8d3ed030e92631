// Subgroup-to-tier allocation proportional to path bandwidth (Eq. 1 of the paper) and its online re-estimation
// (Section 3.3).  Host logic only.
#include <math.h>

#include <vector>

#include "mlpo_internal.h"

using namespace mlpo;

namespace {

// Exact arithmetic on doubles, as far as Eq. 1 needs it: the sign of a sum of products.  A product of two doubles is
// the unevaluated sum of two doubles (the rounded product and its error, which one fused multiply-add yields), and a
// sum of doubles can be kept exactly as a list of non-overlapping components that grows by one with every addend
// (the classical error-free transformations).  The sign of the whole is the sign of its largest component.  Exact as
// long as no product overflows or falls into the subnormal range, i.e. for any bandwidths a machine can have.
struct ExactSum {
    double part[2 * 66 + 4];
    int n = 0;
    void add(double x) {  // components stay ordered by increasing magnitude, zeros are dropped
        int kept = 0;
        for (int i = 0; i < n; ++i) {
            const double s = x + part[i];
            const double bv = s - x;
            const double err = (x - (s - bv)) + (part[i] - bv);
            if (err != 0.0) part[kept++] = err;
            x = s;
        }
        if (x != 0.0) part[kept++] = x;
        n = kept;
    }
    void add_product(double a, double b) {
        const double hi = a * b;
        add(fma(a, b, -hi));
        add(hi);
    }
    int sign() const { return n == 0 ? 0 : (part[n - 1] > 0.0 ? 1 : -1); }
};

// sign(c * sum_{j in live} bw[j] - m * bw[i]): is c at least the proportional share of tier i?
int share_sign(int64_t c, int64_t m, int i, const std::vector<int>& live, const double* bw) {
    ExactSum e;
    for (int j : live) e.add_product((double)c, bw[j]);
    e.add_product(-(double)m, bw[i]);
    return e.sign();
}

// sign(ca / ba - cb / bb) for positive ba, bb.
int finish_time_sign(int32_t ca, double ba, int32_t cb, double bb) {
    ExactSum e;
    e.add_product((double)ca, bb);
    e.add_product(-(double)cb, ba);
    return e.sign();
}

// Eq. 1 over the tiers listed in `live`, for `m` subgroups: ceilings of the proportional shares (the exact ceiling
// of the exact quotient of the doubles: a floating-point estimate, corrected by exact comparisons), then the surplus
// is taken back one subgroup at a time from the tier that would finish last (largest count / bandwidth; among equals
// the one with the lower bandwidth, then the higher index), so that the paths finish as close together as they can.
void proportional(int64_t m, const std::vector<int>& live, const double* bw, int32_t* count) {
    double total = 0.0;
    for (int i : live) total += bw[i];
    int64_t sum = 0;
    for (int i : live) {
        int64_t c = (int64_t)ceil((double)m * bw[i] / total);
        if (c < 0) c = 0;
        if (c > m) c = m;
        while (c < m && share_sign(c, m, i, live, bw) < 0) ++c;
        while (c > 0 && share_sign(c - 1, m, i, live, bw) >= 0) --c;
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
            const int cmp = finish_time_sign(count[i], bw[i], count[worst], bw[worst]);
            if (cmp > 0 || (cmp == 0 && (bw[i] < bw[worst] || (bw[i] == bw[worst] && i > worst)))) worst = i;
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
