// Analytic profile selection on measured numbers (KVServe section 6.1): the bandwidth threshold
// below which a profile pays off (Eq. 5, Theorem 1) and the piecewise-optimal policy over
// x = 1 / bandwidth (Eq. 6, Theorem 2).  Host code only.
//
// A profile is a line cost(x) = 1/s_p + x/cr_p; moving the KV uncompressed is the line
// cost(x) = x (profile -1).  The policy table is the lower envelope of these lines for x >= 0,
// built by sorting by slope and keeping a stack of segments.
#include "../../include/kvc.h"

#include <algorithm>
#include <cmath>
#include <vector>

namespace {

struct Line {
    double a, b;        // intercept 1/s_p, slope 1/cr_p
    double x_from;      // where the line takes over on the envelope
    int32_t profile;
};

bool valid(const kvc_profile &p)
{
    return std::isfinite(p.cr) && std::isfinite(p.s_enc) && std::isfinite(p.s_dec) && p.cr > 0 && p.s_enc > 0 && p.s_dec > 0;
}

}  // namespace

extern "C" double kvc_profile_throughput(const kvc_profile *p)
{
    if (!p || !valid(*p)) return 0.0;
    return 1.0 / (1.0 / p->s_enc + 1.0 / p->s_dec);
}

extern "C" double kvc_benefit_threshold(const kvc_profile *p)
{
    if (!p || !valid(*p)) return 0.0;
    return (1.0 - 1.0 / p->cr) * kvc_profile_throughput(p);
}

extern "C" int kvc_policy_build(const kvc_profile *profiles, int32_t n, kvc_policy_segment *table, int32_t capacity,
                                int32_t *count)
{
    if (n < 0 || (n > 0 && !profiles) || !count || (capacity > 0 && !table) || capacity < 0) return KVC_ERR_ARG;
    std::vector<Line> lines;
    lines.push_back(Line{0.0, 1.0, 0.0, -1});
    for (int32_t i = 0; i < n; ++i) {
        if (!valid(profiles[i])) return KVC_ERR_ARG;
        lines.push_back(Line{1.0 / kvc_profile_throughput(&profiles[i]), 1.0 / profiles[i].cr, 0.0, i});
    }
    // steepest first; among equal slopes only the lowest line can ever be optimal
    std::sort(lines.begin(), lines.end(), [](const Line &l, const Line &r) {
        if (l.b != r.b) return l.b > r.b;
        if (l.a != r.a) return l.a < r.a;
        return l.profile < r.profile;
    });
    std::vector<Line> hull;
    for (Line l : lines) {
        if (!hull.empty() && l.b == hull.back().b) continue;
        double x = 0.0;
        while (!hull.empty()) {
            const Line &top = hull.back();
            x = (l.a - top.a) / (top.b - l.b);          // from here on l is below top
            if (x <= top.x_from) hull.pop_back();       // top is never the lowest
            else break;
        }
        l.x_from = hull.empty() ? 0.0 : x;
        hull.push_back(l);
    }
    *count = (int32_t)hull.size();
    if ((int32_t)hull.size() > capacity) return KVC_ERR_CAPACITY;
    for (size_t i = 0; i < hull.size(); ++i) {
        table[i].x_from = hull[i].x_from;
        table[i].profile = hull[i].profile;
    }
    return KVC_OK;
}

extern "C" int kvc_policy_lookup(const kvc_policy_segment *table, int32_t count, double bandwidth, int32_t *profile,
                                 int32_t *toward_more_bandwidth, int32_t *toward_less_bandwidth)
{
    if (!table || count < 1 || !profile || !(bandwidth > 0)) return KVC_ERR_ARG;
    const double x = 1.0 / bandwidth;
    int32_t lo = 0, hi = count - 1;                     // last segment with x_from <= x
    while (lo < hi) {
        const int32_t mid = (lo + hi + 1) / 2;
        if (table[mid].x_from <= x) lo = mid;
        else hi = mid - 1;
    }
    *profile = table[lo].profile;
    if (toward_more_bandwidth) *toward_more_bandwidth = lo > 0 ? table[lo - 1].profile : table[lo].profile;
    if (toward_less_bandwidth) *toward_less_bandwidth = lo + 1 < count ? table[lo + 1].profile : table[lo].profile;
    return KVC_OK;
}
