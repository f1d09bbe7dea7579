// Groups of compute units from the pair-throughput heatmap (paper Sec. 2.2:
// pairs of SMs that share a memory-side resource are slower together; Fig. 3
// re-arranges the indices so that the groups show).  The paper states no
// algorithm; the rule implemented here is documented at rr_groups_from_heatmap
// in include/randline.h.  Host only.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <vector>

#include "../../include/randline.h"

namespace rr {
int fail(int code, const char *fmt, ...);  // rr_state.hip: records the message for rr_last_error
}
using rr::fail;

namespace {

// Union-find over CU indices.
struct DisjointSets {
    std::vector<uint32_t> parent;
    explicit DisjointSets(uint32_t n) : parent(n) { std::iota(parent.begin(), parent.end(), 0u); }
    uint32_t find(uint32_t x) {
        while (parent[x] != x) {
            parent[x] = parent[parent[x]];
            x = parent[x];
        }
        return x;
    }
    void unite(uint32_t a, uint32_t b) {
        a = find(a);
        b = find(b);
        if (a != b) parent[std::max(a, b)] = std::min(a, b);  // root = smallest member
    }
};

}  // namespace

extern "C" int rr_groups_from_heatmap(const double *T, uint32_t n, const double *singles, double min_gap,
                                      uint16_t *group_out, uint32_t *order_out, uint32_t *n_groups_out,
                                      double *threshold_out) {
    if (!T) return fail(RR_EINVAL, "T is NULL");
    if (n == 0 || n > RR_MAX_CUS) return fail(RR_EINVAL, "n must be in [1, %u] (got %u)", RR_MAX_CUS, n);
    if (!group_out || !order_out || !n_groups_out || !threshold_out) return fail(RR_EINVAL, "an output pointer is NULL");
    if (!(min_gap >= 0.0) || !std::isfinite(min_gap)) return fail(RR_EINVAL, "min_gap must be finite and not negative");
    // Every ratio below must be an ordinary number: a NaN among them would make the sort's order meaningless.
    for (uint32_t a = 0; a < n; ++a)
        for (uint32_t b = a + 1; b < n; ++b) {
            const double t = T[(size_t)a * n + b];
            if (!std::isfinite(t) || t < 0.0)
                return fail(RR_EINVAL, "T[%u][%u] is not a finite, non-negative throughput", a, b);
        }
    if (singles)
        for (uint32_t a = 0; a < n; ++a)
            if (!std::isfinite(singles[a]) || !(singles[a] > 0.0))
                return fail(RR_EINVAL, "singles[%u] is not a finite, positive throughput", a);
    const double nan = std::numeric_limits<double>::quiet_NaN();
    const size_t m = (size_t)n * (n - 1) / 2;
    std::vector<double> ratio(m);
    double top = 0.0;
    if (!singles) {
        for (uint32_t a = 0; a < n; ++a)
            for (uint32_t b = a + 1; b < n; ++b) top = std::max(top, T[(size_t)a * n + b]);
        if (m > 0 && !(top > 0.0)) return fail(RR_EINVAL, "every pair throughput is zero");
    }
    size_t k = 0;
    for (uint32_t a = 0; a < n; ++a)
        for (uint32_t b = a + 1; b < n; ++b, ++k)
            ratio[k] = singles ? T[(size_t)a * n + b] / (singles[a] + singles[b]) : T[(size_t)a * n + b] / top;

    double threshold = nan;
    if (m >= 2) {
        std::vector<double> sorted(ratio);
        std::sort(sorted.begin(), sorted.end());
        double best_gap = -1.0;
        size_t best_i = 0;
        for (size_t i = 0; i + 1 < m; ++i) {
            const double gap = sorted[i + 1] - sorted[i];
            if (gap > best_gap) {  // strict: the first of equal gaps wins
                best_gap = gap;
                best_i = i;
            }
        }
        const double median = (m % 2 == 1) ? sorted[m / 2] : 0.5 * (sorted[m / 2 - 1] + sorted[m / 2]);
        if (!(best_gap < min_gap * median)) threshold = 0.5 * (sorted[best_i] + sorted[best_i + 1]);
    }

    DisjointSets sets(n);
    if (!std::isnan(threshold)) {
        k = 0;
        for (uint32_t a = 0; a < n; ++a)
            for (uint32_t b = a + 1; b < n; ++b, ++k)
                if (ratio[k] < threshold) sets.unite(a, b);
    }
    // number the groups by their smallest member (roots are smallest members, visited ascending)
    std::vector<int32_t> id_of_root(n, -1);
    uint32_t n_groups = 0;
    for (uint32_t u = 0; u < n; ++u) {
        const uint32_t r = sets.find(u);
        if (id_of_root[r] < 0) id_of_root[r] = (int32_t)n_groups++;
        group_out[u] = (uint16_t)id_of_root[r];
    }
    std::vector<uint32_t> order(n);
    std::iota(order.begin(), order.end(), 0u);
    std::stable_sort(order.begin(), order.end(),
                     [&](uint32_t x, uint32_t y) { return group_out[x] < group_out[y]; });
    std::copy(order.begin(), order.end(), order_out);
    *n_groups_out = n_groups;
    *threshold_out = threshold;
    return RR_OK;
}
