// SLO-aware latency control (Algorithm 2 of the paper): host-side threshold controller.  No device code.
#include "../../include/brownout_moe.h"

#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

extern "C" double moe_latency_p90(const double* latencies, size_t n)
{
    if (!latencies || n == 0) return std::numeric_limits<double>::quiet_NaN();
    std::vector<double> v(latencies, latencies + n);
    const size_t rank = (9 * n + 9) / 10;                 // ceil(0.9 n), 1-based
    std::nth_element(v.begin(), v.begin() + (rank - 1), v.end());
    return v[rank - 1];
}

extern "C" double moe_salc_update(double threshold, double latency_p90, const moe_salc_params* p)
{
    const double nan = std::numeric_limits<double>::quiet_NaN();
    if (!p || !std::isfinite(threshold) || !std::isfinite(latency_p90)) return nan;
    if (!std::isfinite(p->slo) || !std::isfinite(p->warning_factor) || !std::isfinite(p->increment) ||
        !std::isfinite(p->shrink_ratio))
        return nan;
    if (p->slo <= 0.0 || p->warning_factor <= 0.0 || p->warning_factor > 1.0 || p->increment < 0.0 ||
        p->shrink_ratio < 0.0 || p->shrink_ratio > 1.0)
        return nan;
    const double warning_line = p->slo * p->warning_factor;
    double t = threshold;
    if (latency_p90 < warning_line) t = threshold + p->increment;
    else if (latency_p90 > p->slo) t = threshold * p->shrink_ratio;
    return std::min(1.0, std::max(0.0, t));
}
