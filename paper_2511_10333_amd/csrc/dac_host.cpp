// Host arithmetic of the Dynamic Alignment Compressor.
//
// Sec. IV-D-1: the inequality that bounds the useful ranks and the linear model
// T_com(r) = eta r; Sec. IV-D-4 / Algorithm 2: stage-aligned ranks; Sec. IV-B:
// iteration sampling rate.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <vector>

#include "edgc.h"

namespace {

bool ascending(const uint32_t* v, uint32_t n)
{
    return std::adjacent_find(v, v + n, [](uint32_t a, uint32_t b) { return a >= b; }) == v + n;
}

}  // namespace

extern "C" int edgc_rank_bounds(const edgc_rank_cost* costs, uint32_t n, double bytes_original,
                                double bandwidth, double r_min_divisor,
                                edgc_rank_bounds_result* out, double* t_com_out)
{
    if (!costs || !out || n == 0) return EDGC_EINVAL;
    if (!std::isfinite(bytes_original) || !std::isfinite(bandwidth) || !std::isfinite(r_min_divisor))
        return EDGC_ENONFINITE;
    if (bytes_original <= 0.0 || bandwidth <= 0.0 || r_min_divisor < 4.0 || r_min_divisor > 6.0)
        return EDGC_EINVAL;
    std::vector<double> total(n);
    for (uint32_t i = 0; i < n; ++i) {
        const edgc_rank_cost& c = costs[i];
        if (!std::isfinite(c.t_compress) || !std::isfinite(c.t_decompress) || !std::isfinite(c.bytes_compressed))
            return EDGC_ENONFINITE;
        if (c.t_compress < 0.0 || c.t_decompress < 0.0 || c.bytes_compressed < 0.0) return EDGC_EINVAL;
        if (c.rank == 0 || (i > 0 && c.rank <= costs[i - 1].rank)) return EDGC_EINVAL;
        total[i] = c.t_compress + c.bytes_compressed / bandwidth + c.t_decompress;
    }
    const double plain = bytes_original / bandwidth;
    // index of the first candidate whose compressed exchange is slower than the plain one
    const auto first_bad = std::find_if(total.begin(), total.end(), [plain](double t) { return t > plain; });
    const size_t n_good = static_cast<size_t>(first_bad - total.begin());
    out->r_max = n_good ? costs[n_good - 1].rank : 0u;
    out->r_min = 0;
    if (out->r_max) {
        const double q = std::ceil(static_cast<double>(out->r_max) / r_min_divisor);
        out->r_min = q < 1.0 ? 1u : static_cast<uint32_t>(q);
    }
    out->t_uncompressed = plain;
    if (t_com_out) std::copy(total.begin(), total.end(), t_com_out);
    return EDGC_OK;
}

extern "C" int edgc_fit_eta(const uint32_t* ranks, const double* t_com, uint32_t n, double* eta,
                            double* mape_percent)
{
    if (!ranks || !t_com || !eta || n == 0) return EDGC_EINVAL;
    double rt = 0.0, rr = 0.0;
    for (uint32_t i = 0; i < n; ++i) {
        if (!std::isfinite(t_com[i])) return EDGC_ENONFINITE;
        if (ranks[i] == 0 || t_com[i] <= 0.0) return EDGC_EINVAL;
        const double r = static_cast<double>(ranks[i]);
        rt += r * t_com[i];
        rr += r * r;
    }
    const double slope = rt / rr;
    *eta = slope;
    if (mape_percent) {
        double acc = 0.0;
        for (uint32_t i = 0; i < n; ++i)
            acc += std::fabs(t_com[i] - slope * static_cast<double>(ranks[i])) / t_com[i];
        *mape_percent = 100.0 * acc / static_cast<double>(n);
    }
    return EDGC_OK;
}

extern "C" int edgc_stage_ranks(uint32_t r_stage1, double t_microback, double eta, uint32_t r_min,
                                uint32_t r_max, const uint32_t* allowed, uint32_t n_allowed,
                                uint32_t n_stages, uint32_t* ranks_out, double* t_com_out)
{
    if (!ranks_out || n_stages == 0) return EDGC_EINVAL;
    if (!std::isfinite(t_microback) || !std::isfinite(eta)) return EDGC_ENONFINITE;
    if (eta <= 0.0 || t_microback < 0.0 || r_min == 0 || r_min > r_max) return EDGC_EINVAL;
    if (n_allowed && (!allowed || !ascending(allowed, n_allowed))) return EDGC_EINVAL;
    const double t_first = eta * static_cast<double>(r_stage1);
    ranks_out[0] = r_stage1;
    for (uint32_t stage = 1; stage < n_stages; ++stage) {
        // stage index `stage` is the paper's stage i = stage + 1, offset i - 1 = stage
        const double want = std::floor((t_first + static_cast<double>(stage) * t_microback) / eta + 1e-9);
        uint32_t r = want >= static_cast<double>(r_max) ? r_max
                   : want <= static_cast<double>(r_min) ? r_min
                                                        : static_cast<uint32_t>(want);
        if (n_allowed) {
            // last allowed value <= r, or the first one when every value is larger
            const uint32_t* above = std::upper_bound(allowed, allowed + n_allowed, r);
            r = above == allowed ? allowed[0] : above[-1];
        }
        ranks_out[stage] = r;
    }
    if (t_com_out)
        for (uint32_t stage = 0; stage < n_stages; ++stage)
            t_com_out[stage] = eta * static_cast<double>(ranks_out[stage]);
    return EDGC_OK;
}

extern "C" int edgc_entropy_due(uint64_t iter_in_window, uint32_t period)
{
    if (period == 0) return EDGC_EINVAL;
    return iter_in_window % period == 0 ? 1 : 0;
}
