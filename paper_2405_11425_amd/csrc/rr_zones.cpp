// Memory zones of an allocation from pair rates of its windows: the paper's pair probe (Sec. 2.2: run the
// access kernel on two units at a time and see which pairs slow each other down) applied to pieces of memory
// instead of compute units.  The rule is documented at rr_zones_from_pair_rates in include/randline.h; the
// measurement that feeds it on a device (rr_detect_zones) is in rr_api.hip.  Host only.
#include <algorithm>
#include <cmath>
#include <cstring>

#include "rr_zones.hpp"

using rr::fail;

namespace rr {

namespace {

// One rate from the caller's function, checked: the rule compares and sorts these values.
int take(rr_pair_rate_fn rate, void *user, uint32_t a, uint32_t b, int again, double *out) {
    double r = 0.0;
    const int rc = rate(a, b, again, user, &r);
    if (rc != RR_OK) return rc;
    if (!std::isfinite(r) || r < 0.0) return fail(RR_EINVAL, "rate(%u, %u) is not a finite, non-negative number", a, b);
    *out = r;
    return RR_OK;
}

double median_of(double *v, uint32_t m) {  // m >= 1; sorts v
    std::sort(v, v + m);
    return (m % 2 == 1) ? v[m / 2] : 0.5 * (v[m / 2 - 1] + v[m / 2]);
}

}  // namespace

int zones_rule(rr_pair_rate_fn rate, void *user, uint32_t n, double min_gap, uint32_t max_zones, uint8_t *zone_out,
               rr_zone_probe_t *details) {
    rr_zone_probe_t d;
    memset(&d, 0, sizeof d);
    int rc;
    // step 1, first half: a window paired with itself certainly shares a zone with itself
    uint32_t picks[4] = {0, n / 3, 2 * n / 3, n - 1};
    std::sort(picks, picks + 4);
    const uint32_t n_picks = (uint32_t)(std::unique(picks, picks + 4) - picks);
    double same = 0.0, r;
    for (uint32_t i = 0; i < n_picks; ++i) {
        if ((rc = take(rate, user, picks[i], picks[i], 0, &r)) != RR_OK) return rc;
        same = std::max(same, r);
    }
    // step 2: window 0 with every other one
    for (uint32_t b = 1; b < n; ++b)
        if ((rc = take(rate, user, 0, b, 0, &d.row[b])) != RR_OK) return rc;
    // step 1, second half
    for (uint32_t i = 0; i < n_picks; ++i) {
        if ((rc = take(rate, user, picks[i], picks[i], 0, &r)) != RR_OK) return rc;
        same = std::max(same, r);
    }
    d.pair_rates = 2 * n_picks + (n - 1);
    // step 3: one cluster or two in the first row?
    double low[RR_MAX_ZONE_WINDOWS];
    uint32_t n_low = 0;
    for (uint32_t b = 1; b < n; ++b)
        if (d.row[b] < same * (1.0 - min_gap)) low[n_low++] = d.row[b];
    double cut = same * (1.0 - min_gap);
    if (n_low >= 2) {
        const double med = median_of(low, n_low);
        if (med < same * (1.0 - 1.4 * min_gap)) cut = 0.5 * (same + med);
    }
    const double band = 0.25 * (same - cut);
    d.same = same;
    d.cut = cut;
    d.band = band;

    // step 4: do a and b run together?  `first` is the pair's rate if it has been measured already.
    auto together = [&](uint32_t a, uint32_t b, const double *first, bool *yes) -> int {
        double v;
        if (first) {
            v = *first;
        } else {
            int rc2 = take(rate, user, a, b, 0, &v);
            if (rc2 != RR_OK) return rc2;
            d.pair_rates++;
        }
        if (std::fabs(v - cut) < band) {
            double again;
            int rc2 = take(rate, user, a, b, 1, &again);
            if (rc2 != RR_OK) return rc2;
            d.retakes++;
            v = std::max(v, again);
        }
        *yes = v >= cut;
        return RR_OK;
    };

    // step 5: greedy assignment by representative
    int zone[RR_MAX_ZONE_WINDOWS];
    for (uint32_t b = 0; b < n; ++b) zone[b] = -1;
    uint32_t n_zones = 0;
    for (;;) {
        uint32_t ref = 0;
        while (ref < n && zone[ref] != -1) ++ref;
        if (ref == n) break;
        if (n_zones == max_zones) {  // step 6
            d.gave_up = 1;
            for (uint32_t b = 0; b < n; ++b) zone[b] = 0;
            n_zones = 1;
            break;
        }
        zone[ref] = (int)n_zones;
        for (uint32_t b = ref + 1; b < n; ++b) {
            if (zone[b] != -1) continue;
            bool yes = false;
            if ((rc = together(ref, b, ref == 0 ? &d.row[b] : nullptr, &yes)) != RR_OK) return rc;
            if (yes) zone[b] = (int)n_zones;
        }
        n_zones++;
    }
    for (uint32_t b = 0; b < n; ++b) d.before_merging[b] = (uint8_t)zone[b];
    // step 7: zones whose first windows run together after all (their first comparison was taken while the
    // process was still starting up, say) are one zone
    if (!d.gave_up) {
        uint32_t first_of[RR_MAX_ZONES], joined[RR_MAX_ZONES];
        for (uint32_t z = 0; z < n_zones; ++z) {
            joined[z] = z;
            first_of[z] = 0;
            while (zone[first_of[z]] != (int)z) ++first_of[z];
        }
        for (uint32_t zb = 1; zb < n_zones; ++zb)
            for (uint32_t za = 0; za < zb; ++za) {
                if (joined[za] != za) continue;
                d.merge_rates++;
                if ((rc = take(rate, user, first_of[za], first_of[zb], 1, &r)) != RR_OK) return rc;
                if (r >= cut) {
                    joined[zb] = za;
                    break;
                }
            }
        int new_id[RR_MAX_ZONES];
        for (uint32_t z = 0; z < n_zones; ++z) new_id[z] = -1;
        uint32_t n_after = 0;
        for (uint32_t b = 0; b < n; ++b) {  // renumber in order of first appearance
            const uint32_t root = joined[zone[b]];
            if (new_id[root] < 0) new_id[root] = (int)n_after++;
            zone[b] = new_id[root];
        }
        n_zones = n_after;
    }
    d.n_zones = n_zones;
    for (uint32_t b = 0; b < n; ++b) zone_out[b] = (uint8_t)zone[b];
    if (details) *details = d;
    return RR_OK;
}

int check_zone_rule_args(uint32_t n, double min_gap, uint32_t max_zones, const void *zone_out) {
    if (n == 0 || n > RR_MAX_ZONE_WINDOWS) return fail(RR_EINVAL, "n_windows must be in [1, %u] (got %u)", RR_MAX_ZONE_WINDOWS, n);
    if (!std::isfinite(min_gap) || !(min_gap > 0.0) || !(min_gap < 0.5))
        return fail(RR_EINVAL, "min_gap must lie in (0, 0.5)");
    if (max_zones == 0 || max_zones > RR_MAX_ZONES) return fail(RR_EINVAL, "max_zones must be in [1, %u]", RR_MAX_ZONES);
    if (!zone_out) return fail(RR_EINVAL, "zone_of_window_out is NULL");
    return RR_OK;
}

}  // namespace rr

extern "C" int rr_zones_from_pair_rates(rr_pair_rate_fn rate, void *user, uint32_t n_windows, double min_gap,
                                        uint32_t max_zones, uint8_t *zone_of_window_out, rr_zone_probe_t *details_out) {
    if (!rate) return fail(RR_EINVAL, "rate is NULL");
    int rc = rr::check_zone_rule_args(n_windows, min_gap, max_zones, zone_of_window_out);
    if (rc != RR_OK) return rc;
    uint8_t zone[RR_MAX_ZONE_WINDOWS];  // outputs are written on success only
    rr_zone_probe_t d;
    rc = rr::zones_rule(rate, user, n_windows, min_gap, max_zones, zone, &d);
    if (rc != RR_OK) return rc;
    memcpy(zone_of_window_out, zone, n_windows);
    if (details_out) *details_out = d;
    return RR_OK;
}
