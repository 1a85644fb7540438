// Entropy window -> compression rank (host only).
//
// CQM of the paper: Lemma 1 (closed-form Marchenko-Pastur CDF), Theorem 1
// (g(r; m, n) from eigenvalue quantiles), Theorem 3 (r1 = g^-1(e^{H0-H1} g(r0)))
// and the window rule of Sec. IV-D: adaptive warm-up (IV-D-2) and Algorithm 1
// with the step limit of Constraint 2.
#include <algorithm>
#include <cmath>
#include <map>
#include <memory>
#include <mutex>
#include <utility>
#include <vector>

#include "edgc.h"

namespace {

// Marchenko-Pastur law of the eigenvalues of A A^T for an mm x nn matrix
// (mm <= nn) with unit-variance entries, support [a, b].
class MarchenkoPastur {
public:
    MarchenkoPastur(uint32_t m, uint32_t n)
        : mm_(std::min(m, n)), nn_(std::max(m, n))
    {
        const double sm = std::sqrt(static_cast<double>(mm_)), sn = std::sqrt(static_cast<double>(nn_));
        a_ = (sn - sm) * (sn - sm);
        b_ = (sn + sm) * (sn + sm);
        gm_ = std::sqrt(a_ * b_);
    }
    // Lemma 1:  F = [ -2 sqrt(ab) atan(sqrt(b(l-a) / (a(b-l)))) + (a+b) asin(sqrt((l-a)/(b-a)))
    //                 + sqrt((l-a)(b-l)) ] / (2 pi mm)
    double cdf(double l) const
    {
        if (l <= a_) return 0.0;
        if (l >= b_) return 1.0;
        const double up = l - a_, dn = b_ - l;
        double bracket = (a_ + b_) * std::asin(std::sqrt(up / (b_ - a_))) + std::sqrt(up * dn);
        if (gm_ > 0.0) bracket -= 2.0 * gm_ * std::atan2(std::sqrt(b_ * up), std::sqrt(a_ * dn));
        return bracket / (2.0 * M_PI * static_cast<double>(mm_));
    }
    // density of the same law: dF/dl = sqrt((l-a)(b-l)) / (2 pi mm l)
    double pdf(double l) const
    {
        if (l <= a_ || l >= b_) return 0.0;
        return std::sqrt((l - a_) * (b_ - l)) / (2.0 * M_PI * static_cast<double>(mm_) * l);
    }
    // inverse CDF on [from, b]; `from` must satisfy cdf(from) <= p.  Newton steps from `from`,
    // kept inside a bracket that every evaluation tightens; a step that leaves the bracket
    // (the density vanishes at both ends of the support) is replaced by its mid-point.
    double quantile(double p, double from) const
    {
        double lo = std::max(from, a_), hi = b_;
        double x = lo;
        for (int it = 0; it < 200; ++it) {
            const double f = cdf(x) - p;
            (f < 0.0 ? lo : hi) = x;
            const double d = pdf(x);
            double nx = d > 0.0 ? x - f / d : lo + 0.5 * (hi - lo);
            if (!(nx > lo && nx < hi)) nx = lo + 0.5 * (hi - lo);
            if (!(nx > lo && nx < hi)) break;             // the bracket is one rounding step wide
            if (std::fabs(nx - x) <= 4e-16 * std::fabs(nx)) { x = nx; break; }
            x = nx;
        }
        return x;
    }
    uint32_t small() const { return mm_; }
    double a() const { return a_; }

private:
    uint32_t mm_, nn_;
    double a_, b_, gm_;
};

// g[r] for r = 0..mm: Theorem 1 with the mid-point quantiles (k - 1/2)/mm in place
// of uniform random draws, i.e. the expectation of the sampled eigenvalues.
std::shared_ptr<const std::vector<double>> error_table(uint32_t m, uint32_t n)
{
    static std::mutex mu;
    static std::map<std::pair<uint32_t, uint32_t>, std::shared_ptr<const std::vector<double>>> cache;
    const auto key = std::make_pair(std::min(m, n), std::max(m, n));
    {
        std::lock_guard<std::mutex> lk(mu);
        auto it = cache.find(key);
        if (it != cache.end()) return it->second;
    }
    MarchenkoPastur mp(m, n);
    const uint32_t mm = mp.small();
    std::vector<double> lam(mm);
    double prev = mp.a();
    for (uint32_t k = 0; k < mm; ++k) {                 // ascending: reuse the last root as bracket
        lam[k] = mp.quantile((static_cast<double>(k) + 0.5) / static_cast<double>(mm), prev);
        prev = lam[k];
    }
    auto g = std::make_shared<std::vector<double>>(static_cast<size_t>(mm) + 1, 0.0);
    double tail = 0.0;                                   // sum of the (mm - r) smallest eigenvalues
    for (uint32_t r = mm; r-- > 0;) {
        tail += lam[mm - 1 - r];
        (*g)[r] = std::sqrt(tail);
    }
    std::lock_guard<std::mutex> lk(mu);
    if (cache.size() > 64) cache.clear();
    cache[key] = g;
    return g;
}

}  // namespace

extern "C" int edgc_select_rank(edgc_rank_state* st, const double* H_window, uint32_t k,
                                uint64_t iters_in_window, const edgc_rank_params* prm,
                                edgc_rank_decision* out)
{
    if (!st || !H_window || !prm || !out || k == 0) return EDGC_EINVAL;
    const uint32_t mm = std::min(prm->m, prm->n);
    // rank 0 is the warm-up answer: 1 <= r_min <= r_max <= min(m, n)
    if (mm == 0 || prm->r_min == 0 || prm->r_max > mm || prm->r_min > prm->r_max) return EDGC_EINVAL;
    const uint32_t r_ref = prm->r_ref ? prm->r_ref : prm->r_max;
    if (r_ref > mm) return EDGC_EINVAL;
    if (prm->n_allowed && !prm->allowed) return EDGC_EINVAL;
    for (uint32_t i = 1; i < prm->n_allowed; ++i)
        if (prm->allowed[i] <= prm->allowed[i - 1]) return EDGC_EINVAL;
    // the allowed ranks inside the bounds, [lo_ok, hi_ok): the only ones ever emitted
    const uint32_t* const lo_ok = std::lower_bound(prm->allowed, prm->allowed + prm->n_allowed, prm->r_min);
    const uint32_t* const hi_ok = std::upper_bound(prm->allowed, prm->allowed + prm->n_allowed, prm->r_max);
    if (prm->n_allowed && lo_ok >= hi_ok) return EDGC_EINVAL;

    double sum = 0.0;
    for (uint32_t i = 0; i < k; ++i) {
        if (!std::isfinite(H_window[i])) return EDGC_ENONFINITE;
        sum += H_window[i];
    }
    const double H_mean = sum / static_cast<double>(k);      // window average (Sec. IV-D-3)
    st->iters_seen += iters_in_window;

    *out = edgc_rank_decision{};
    out->H_mean = H_mean;

    if (!st->have_ref) {                                     // initial gradients anchor Theorem 3
        st->have_ref = 1;
        st->compressing = 0;
        st->H_ref = H_mean;
        st->r_prev = static_cast<double>(r_ref);
        out->r_unclamped = static_cast<double>(r_ref);
        return EDGC_OK;
    }

    // Theorem 3 at fixed absolute error: g(r_new) <= exp(H_ref - H_mean) * g(r_ref)
    const auto g = error_table(prm->m, prm->n);
    const double budget = std::exp(st->H_ref - H_mean) * (*g)[r_ref];
    // g is strictly decreasing: first index whose value does not exceed the budget
    const auto it = std::partition_point(g->begin(), g->end(), [budget](double v) { return v > budget; });
    const uint32_t r_new = static_cast<uint32_t>(it - g->begin());
    out->r_unclamped = static_cast<double>(r_new);

    if (!st->compressing) {                                  // adaptive warm-up (Sec. IV-D-2)
        const bool stabilised = r_new < prm->r_max;
        const bool long_enough = static_cast<double>(st->iters_seen) >=
                                 prm->min_warmup_frac * static_cast<double>(prm->total_iters);
        if (!(stabilised && long_enough)) return EDGC_OK;    // rank stays 0
        st->compressing = 1;
        st->r_prev = static_cast<double>(r_ref);
    }

    // Algorithm 1: bounded move (Constraint 2), then the rank bounds
    const double want = static_cast<double>(r_new), s = static_cast<double>(prm->step_limit);
    double r = want;
    if (want - st->r_prev > s) r = st->r_prev + s;
    else if (st->r_prev - want > s) r = st->r_prev - s;
    r = std::max(static_cast<double>(prm->r_min), std::min(static_cast<double>(prm->r_max), r));
    st->r_prev = r;

    uint32_t rank = static_cast<uint32_t>(r);
    if (prm->n_allowed) {
        // smallest allowed rank >= the state that stays within r_max (Sec. IV-D-1: from r_max on
        // compression no longer pays), else the largest allowed rank inside the bounds
        const uint32_t* p = std::lower_bound(lo_ok, hi_ok, rank);
        rank = (p == hi_ok) ? hi_ok[-1] : *p;
    }
    out->rank = rank;
    out->T_com = prm->eta * static_cast<double>(rank);       // T_com(r) = eta r (Sec. IV-D-1)
    return EDGC_OK;
}
