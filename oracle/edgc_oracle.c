/*
 * EDGC CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 * See edgc_oracle.h for the scope, the readings R1..R10 of the paper and the
 * list of pins.  Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC.
 * fp32 storage, fp64 accumulation, no code shared with the HIP sources.
 */
#include "edgc_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ------------------------------------------------------------------------ */
/* small exact helpers                                                       */
/* ------------------------------------------------------------------------ */

/* How many threads the loops over independent outputs use from now on (n >= 1);
 * no effect on any result.  Lets the benchmark time the oracle on one core and on all. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* bf16 <-> fp32.  bf16 is the upper 16 bits of an IEEE binary32; widening is
 * exact, narrowing is round-to-nearest-even on the dropped 16 bits. */
float oracle_bf16_to_f32(uint16_t h)
{
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

uint16_t oracle_f32_to_bf16(float x)
{
    uint32_t u;
    memcpy(&u, &x, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u)          /* NaN: keep it a NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

static float round_through_bf16(float x)
{
    return oracle_bf16_to_f32(oracle_f32_to_bf16(x));
}

/* A fixed 64-bit integer mixer (the splitmix64 output function applied to
 * seed + golden-ratio * (ctr + 1)).  Both sides of the parity tests write it
 * out independently; it is the only "random" draw the method makes (R2) apart
 * from the initial Q. */
uint64_t oracle_mix64(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * (ctr + 1ull);
    z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27; z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

/* ------------------------------------------------------------------------ */
/* GDS: gradient sampling rate beta (Sec. IV-B), reading R2                  */
/* ------------------------------------------------------------------------ */

uint64_t oracle_sample_slot(uint64_t seed, uint64_t step, uint64_t stride)
{
    return stride ? oracle_mix64(seed, step) % stride : 0;
}

uint64_t oracle_sample_indices(uint64_t n, uint64_t stride, uint32_t chunk,
                               uint64_t seed, uint64_t step, uint64_t* idx, uint64_t cap)
{
    if (stride == 0 || chunk == 0) return 0;
    const uint64_t slot = oracle_sample_slot(seed, step, stride);
    uint64_t cnt = 0;
    /* chunk c = floor(i / chunk) is sampled iff c mod stride == slot */
    for (uint64_t c = slot; c * (uint64_t)chunk < n; c += stride) {
        for (uint64_t e = 0; e < chunk; ++e) {
            uint64_t i = c * (uint64_t)chunk + e;
            if (i >= n) break;
            if (idx && cnt < cap) idx[cnt] = i;
            ++cnt;
        }
    }
    return cnt;
}

static float load_as_f32(const void* p, int dtype, uint64_t i)
{
    if (dtype == ORACLE_BF16) return oracle_bf16_to_f32(((const uint16_t*)p)[i]);
    return ((const float*)p)[i];
}

/* ------------------------------------------------------------------------ */
/* Entropy of the sample: Definition 1 / Eq. (1) estimated by a histogram    */
/* (readings R1, R3)                                                          */
/* ------------------------------------------------------------------------ */

int oracle_entropy(const void* grad, int dtype, uint64_t n, uint64_t stride, uint32_t chunk,
                   uint64_t seed, uint64_t step, uint32_t bins, const float* range_lo_hi,
                   oracle_entropy_result* out, uint64_t* counts)
{
    if (!grad || !out || stride == 0 || chunk == 0 || bins == 0 || bins > (1u << 24))
        return ORACLE_EINVAL;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_EINVAL;
    if (range_lo_hi && !(range_lo_hi[0] <= range_lo_hi[1])) return ORACLE_EINVAL;

    uint64_t* own = NULL;
    if (!counts) {
        own = (uint64_t*)calloc(bins, sizeof(uint64_t));
        if (!own) return ORACLE_ENOMEM;
        counts = own;
    } else {
        memset(counts, 0, (size_t)bins * sizeof(uint64_t));
    }

    const uint64_t slot = oracle_sample_slot(seed, step, stride);

    /* pass 1: count, skip non-finite, range of the finite sample */
    uint64_t n_sampled = 0, n_nonfinite = 0;
    float lo = INFINITY, hi = -INFINITY;
    for (uint64_t c = slot; c * (uint64_t)chunk < n; c += stride) {
        for (uint64_t e = 0; e < chunk; ++e) {
            uint64_t i = c * (uint64_t)chunk + e;
            if (i >= n) break;
            float x = load_as_f32(grad, dtype, i);
            ++n_sampled;
            if (!isfinite(x)) { ++n_nonfinite; continue; }
            if (x < lo) lo = x;
            if (x > hi) hi = x;
        }
    }
    memset(out, 0, sizeof *out);
    out->n_sampled = n_sampled;
    out->n_nonfinite = n_nonfinite;
    const uint64_t n_used = n_sampled - n_nonfinite;
    if (n_used == 0) {
        out->H_bits = NAN; out->h_diff_nats = NAN; out->lo = NAN; out->hi = NAN;
        free(own);
        return ORACLE_ENONFINITE;
    }
    if (range_lo_hi) { lo = range_lo_hi[0]; hi = range_lo_hi[1]; }
    out->lo = lo;
    out->hi = hi;

    /* pass 2: equal-width bins over [lo, hi]; fp32, separately rounded ops */
    const float w = hi - lo;
    const float fbins = (float)bins;
    const float scale = (w > 0.0f) ? fbins / w : 0.0f;
    for (uint64_t c = slot; c * (uint64_t)chunk < n; c += stride) {
        for (uint64_t e = 0; e < chunk; ++e) {
            uint64_t i = c * (uint64_t)chunk + e;
            if (i >= n) break;
            float x = load_as_f32(grad, dtype, i);
            if (!isfinite(x)) continue;
            uint32_t b = 0;
            if (w > 0.0f) {
                float t = x - lo;          /* rounded subtract        */
                float u = t * scale;       /* rounded multiply, no FMA */
                if (u >= fbins)     b = bins - 1;
                else if (u >= 0.0f) b = (uint32_t)u;   /* truncation */
                else                b = 0;
            }
            counts[b] += 1;
        }
    }

    /* H = -sum p_i log2 p_i with p_i = c_i / n  ==  log2 n - (1/n) sum c_i log2 c_i */
    double s = 0.0;
    for (uint32_t b = 0; b < bins; ++b)
        if (counts[b] > 0) s += (double)counts[b] * log2((double)counts[b]);
    double H = log2((double)n_used) - s / (double)n_used;
    if (H < 0.0) H = 0.0;                 /* rounding can leave -1e-17 for a single bin */
    out->H_bits = H;
    /* histogram estimate of Eq. (1): -sum p_i ln(p_i / width) = H ln 2 + ln width */
    out->h_diff_nats = (w > 0.0f) ? H * log(2.0) + log((double)w / (double)bins) : -INFINITY;
    free(own);
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* CQM: Lemma 1 (Marchenko-Pastur CDF), Theorem 1 (g), Theorem 3, and the     */
/* window rule of Algorithm 1 with the warm-up of Sec. IV-D-2                 */
/* ------------------------------------------------------------------------ */

/* Lemma 1 with m' = min(m,n), n' = max(m,n) (reading R4): the prefactor
 * 1/(2 pi m') normalises the bracket to 1 at lambda = b only for m' <= n'. */
double oracle_mp_cdf(double lambda, uint32_t m, uint32_t n)
{
    const double mm = (double)(m < n ? m : n), nn = (double)(m < n ? n : m);
    const double a = (sqrt(nn) - sqrt(mm)) * (sqrt(nn) - sqrt(mm));
    const double b = (sqrt(nn) + sqrt(mm)) * (sqrt(nn) + sqrt(mm));
    if (lambda <= a) return 0.0;
    if (lambda >= b) return 1.0;
    const double pi = 3.14159265358979323846;
    /* arctan( sqrt( b (l-a) / (a (b-l)) ) ) written with atan2 so a = 0 is fine */
    double t1 = -2.0 * sqrt(a * b) * atan2(sqrt(b * (lambda - a)), sqrt(a * (b - lambda)));
    double t2 = (a + b) * asin(sqrt((lambda - a) / (b - a)));
    double t3 = sqrt((lambda - a) * (b - lambda));
    return (t1 + t2 + t3) / (2.0 * pi * mm);
}

double oracle_mp_quantile(double p, uint32_t m, uint32_t n)
{
    const double mm = (double)(m < n ? m : n), nn = (double)(m < n ? n : m);
    double lo = (sqrt(nn) - sqrt(mm)) * (sqrt(nn) - sqrt(mm));
    double hi = (sqrt(nn) + sqrt(mm)) * (sqrt(nn) + sqrt(mm));
    if (p <= 0.0) return lo;
    if (p >= 1.0) return hi;
    for (int it = 0; it < 200; ++it) {
        double mid = 0.5 * (lo + hi);
        if (mid == lo || mid == hi) break;
        if (oracle_mp_cdf(mid, m, n) < p) lo = mid; else hi = mid;
    }
    return 0.5 * (lo + hi);
}

/* Theorem 1 with deterministic mid-point quantiles in place of the random
 * draws of step (c) (reading R4):  g(r) = sqrt( sum of the m'-r smallest
 * sampled eigenvalues ). */
int64_t oracle_g_table(uint32_t m, uint32_t n, double* g)
{
    const uint32_t mm = m < n ? m : n;
    if (mm == 0 || !g) return -1;
    double* lam = (double*)malloc((size_t)mm * sizeof(double));
    if (!lam) return -1;
    #pragma omp parallel for schedule(static)
    for (int64_t k = 1; k <= (int64_t)mm; ++k)
        lam[k - 1] = oracle_mp_quantile(((double)k - 0.5) / (double)mm, m, n);
    /* quantiles are ascending in k: the m'-r smallest are lam[0 .. m'-r) */
    double pre = 0.0;
    g[mm] = 0.0;
    for (uint32_t cnt = 1; cnt <= mm; ++cnt) {
        pre += lam[cnt - 1];
        g[mm - cnt] = sqrt(pre);
    }
    free(lam);
    return (int64_t)mm;
}

int oracle_select_rank(oracle_rank_state* st, const double* H_window, uint32_t k,
                       uint64_t iters_in_window, const oracle_rank_params* prm,
                       oracle_rank_decision* out)
{
    if (!st || !H_window || !prm || !out || k == 0) return ORACLE_EINVAL;
    const uint32_t mm = prm->m < prm->n ? prm->m : prm->n;
    /* rank 0 is the warm-up answer, so the lower bound is at least 1 */
    if (mm == 0 || prm->r_min == 0 || prm->r_max > mm || prm->r_min > prm->r_max)
        return ORACLE_EINVAL;
    const uint32_t r_ref = prm->r_ref ? prm->r_ref : prm->r_max;
    if (r_ref > mm) return ORACLE_EINVAL;
    for (uint32_t i = 0; i < k; ++i) if (!isfinite(H_window[i])) return ORACLE_ENONFINITE;
    for (uint32_t i = 1; i < prm->n_allowed; ++i)
        if (prm->allowed[i] <= prm->allowed[i - 1]) return ORACLE_EINVAL;
    if (prm->allowed && prm->n_allowed) {           /* R7: some allowed rank must lie in the bounds */
        int inside = 0;
        for (uint32_t i = 0; i < prm->n_allowed; ++i)
            if (prm->allowed[i] >= prm->r_min && prm->allowed[i] <= prm->r_max) inside = 1;
        if (!inside) return ORACLE_EINVAL;
    }

    /* window-mean entropy (Sec. IV-D-3) */
    double Hm = 0.0;
    for (uint32_t i = 0; i < k; ++i) Hm += H_window[i];
    Hm /= (double)k;
    st->iters_seen += iters_in_window;

    memset(out, 0, sizeof *out);
    out->H_mean = Hm;

    if (!st->have_ref) {
        /* first window: the initial gradients fix the reference (R6) */
        st->have_ref = 1;
        st->H_ref = Hm;
        st->r_prev = (double)r_ref;
        st->compressing = 0;
        out->rank = 0;
        out->r_unclamped = (double)r_ref;
        return ORACLE_OK;
    }

    double* g = (double*)malloc(((size_t)mm + 1) * sizeof(double));
    if (!g) return ORACLE_ENOMEM;
    oracle_g_table(prm->m, prm->n, g);

    /* Theorem 3: r1 = g^{-1}( e^{H0 - H1} g(r0) ), g^{-1} by R5 */
    const double target = exp(st->H_ref - Hm) * g[r_ref];
    uint32_t r_new = mm;
    for (uint32_t r = 0; r <= mm; ++r) if (g[r] <= target) { r_new = r; break; }
    free(g);
    out->r_unclamped = (double)r_new;

    /* adaptive warm-up (Sec. IV-D-2): no compression until r_new < r_max and
     * at least min_warmup_frac of all iterations have passed */
    if (!st->compressing) {
        const double need = prm->min_warmup_frac * (double)prm->total_iters;
        if (r_new < prm->r_max && (double)st->iters_seen >= need) {
            st->compressing = 1;
            st->r_prev = (double)r_ref;          /* compression starts at the reference rank */
        } else {
            out->rank = 0;
            return ORACLE_OK;
        }
    }

    /* Algorithm 1: step limit s (Constraint 2), then clamp to the bounds */
    const double s = (double)prm->step_limit;
    double r = (double)r_new;
    if (fabs(r - st->r_prev) > s) r = (r > st->r_prev) ? st->r_prev + s : st->r_prev - s;
    if (r > (double)prm->r_max) r = (double)prm->r_max;
    if (r < (double)prm->r_min) r = (double)prm->r_min;
    st->r_prev = r;

    uint32_t rank = (uint32_t)r;
    if (prm->allowed && prm->n_allowed) {
        /* R7: snap up, but never past r_max (Sec. IV-D-1: from r_max on compression no
         * longer pays, and Algorithm 1 ends with the clamp to [r_min, r_max]): when no
         * allowed rank lies in [rank, r_max], the largest allowed rank <= r_max. */
        uint32_t up = 0, below = 0;
        for (uint32_t i = 0; i < prm->n_allowed; ++i) {
            const uint32_t a = prm->allowed[i];
            if (a < prm->r_min || a > prm->r_max) continue;
            if (a >= rank && !up) up = a;
            if (a < rank) below = a;
        }
        rank = up ? up : below;
    }
    out->rank = rank;
    out->T_com = prm->eta * (double)rank;           /* T_com(r) = eta r, Sec. IV-D-1 */
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------ */
/* Low-rank compressor with error feedback (readings R8, R9, R10)            */
/* ------------------------------------------------------------------------ */

/* Seeded N(0,1) start for Q: column c of row j is a pure function of
 * (seed, j, c), so growing the rank never changes existing columns.
 * Box-Muller on two 53-bit uniforms taken from mix64 at counters 2k, 2k+1,
 * k = j * 2^32 + c. */
void oracle_init_q(float* Q, uint32_t n, uint32_t ldq, uint32_t col_begin, uint32_t col_end,
                   uint64_t seed)
{
    const double two_pi = 6.28318530717958647692;
    for (uint32_t j = 0; j < n; ++j) {
        for (uint32_t c = col_begin; c < col_end; ++c) {
            uint64_t k = ((uint64_t)j << 32) | (uint64_t)c;
            uint64_t z1 = oracle_mix64(seed, 2ull * k);
            uint64_t z2 = oracle_mix64(seed, 2ull * k + 1ull);
            double u1 = ((double)(z1 >> 11) + 0.5) * (1.0 / 9007199254740992.0);
            double u2 = (double)(z2 >> 11) * (1.0 / 9007199254740992.0);
            Q[(size_t)j * ldq + c] = (float)(sqrt(-2.0 * log(u1)) * cos(two_pi * u2));
        }
    }
}

/* P = D * Q   (m x n) * (n x r); fp64 accumulation over j = 0..n-1 in order */
static void contract_P(const float* D, uint32_t m, uint32_t n, const float* Qop, uint32_t r,
                       int round_d, float* P, uint32_t ldp)
{
    #pragma omp parallel
    {
        double* acc = (double*)malloc((size_t)r * sizeof(double));
        #pragma omp for schedule(static)
        for (int64_t i = 0; i < (int64_t)m; ++i) {
            for (uint32_t c = 0; c < r; ++c) acc[c] = 0.0;
            const float* drow = D + (size_t)i * n;
            for (uint32_t j = 0; j < n; ++j) {
                float df = round_d ? round_through_bf16(drow[j]) : drow[j];
                double d = (double)df;
                const float* q = Qop + (size_t)j * r;
                for (uint32_t c = 0; c < r; ++c) acc[c] += d * (double)q[c];
            }
            for (uint32_t c = 0; c < r; ++c) P[(size_t)i * ldp + c] = (float)acc[c];
        }
        free(acc);
    }
}

/* Q = D^T * Pop   (n x m) * (m x r); fp64 accumulation over i = 0..m-1 in order.
 * Threads own disjoint ranges of JB columns of D and keep the JB * r sums of their
 * range side by side, so that D is read along its rows; every (j, c) sum is still
 * the plain sequential sum over i, and the result does not depend on JB. */
static void contract_Q(const float* D, uint32_t m, uint32_t n, const float* Pop, uint32_t r,
                       int round_d, float* Q, uint32_t ldq)
{
    const uint32_t JB = 64;
    #pragma omp parallel
    {
        double* acc = (double*)malloc((size_t)JB * r * sizeof(double));
        #pragma omp for schedule(static)
        for (int64_t jb = 0; jb < (int64_t)((n + JB - 1) / JB); ++jb) {
            const uint32_t j0 = (uint32_t)jb * JB;
            const uint32_t j1 = (j0 + JB < n) ? j0 + JB : n;
            for (size_t t = 0; t < (size_t)JB * r; ++t) acc[t] = 0.0;
            for (uint32_t i = 0; i < m; ++i) {
                const float* p = Pop + (size_t)i * r;
                for (uint32_t j = j0; j < j1; ++j) {
                    float df = D[(size_t)i * n + j];
                    if (round_d) df = round_through_bf16(df);
                    double d = (double)df;
                    double* a = acc + (size_t)(j - j0) * r;
                    for (uint32_t c = 0; c < r; ++c) a[c] += d * (double)p[c];
                }
            }
            for (uint32_t j = j0; j < j1; ++j)
                for (uint32_t c = 0; c < r; ++c)
                    Q[(size_t)j * ldq + c] = (float)acc[(size_t)(j - j0) * r + c];
        }
        free(acc);
    }
}

/* Modified Gram-Schmidt in fp64 on the columns of P (m x r, leading dim ldp);
 * the result has orthonormal columns and R = P^T_hat P has a positive diagonal. */
static int orthonormalise(float* P, uint32_t m, uint32_t r, uint32_t ldp)
{
    double* V = (double*)malloc((size_t)m * r * sizeof(double));   /* column-major */
    if (!V) return ORACLE_ENOMEM;
    double fro2 = 0.0;
    for (uint32_t i = 0; i < m; ++i)
        for (uint32_t c = 0; c < r; ++c) {
            double v = (double)P[(size_t)i * ldp + c];
            V[(size_t)c * m + i] = v;
            fro2 += v * v;
        }
    const double tiny = 1e-30 * sqrt(fro2);
    for (uint32_t j = 0; j < r; ++j) {
        double* vj = V + (size_t)j * m;
        for (uint32_t k = 0; k < j; ++k) {              /* one projection at a time */
            const double* vk = V + (size_t)k * m;
            double dot = 0.0;
            for (uint32_t i = 0; i < m; ++i) dot += vk[i] * vj[i];
            for (uint32_t i = 0; i < m; ++i) vj[i] -= dot * vk[i];
        }
        double nrm2 = 0.0;
        for (uint32_t i = 0; i < m; ++i) nrm2 += vj[i] * vj[i];
        double nrm = sqrt(nrm2);
        if (!(nrm > tiny)) { for (uint32_t i = 0; i < m; ++i) vj[i] = 0.0; }
        else               { for (uint32_t i = 0; i < m; ++i) vj[i] /= nrm; }
    }
    for (uint32_t i = 0; i < m; ++i)
        for (uint32_t c = 0; c < r; ++c)
            P[(size_t)i * ldp + c] = (float)V[(size_t)c * m + i];
    free(V);
    return ORACLE_OK;
}

/* dense copy (optionally rounded through bf16) of an (rows x r) factor */
static float* factor_operand(const float* F, uint32_t rows, uint32_t ld, uint32_t r, int round)
{
    float* o = (float*)malloc((size_t)rows * r * sizeof(float));
    if (!o) return NULL;
    for (uint32_t i = 0; i < rows; ++i)
        for (uint32_t c = 0; c < r; ++c) {
            float v = F[(size_t)i * ld + c];
            o[(size_t)i * r + c] = round ? round_through_bf16(v) : v;
        }
    return o;
}

int oracle_compress(const void* grad, int dtype, uint32_t m, uint32_t n, uint64_t ld,
                    float* residual, int residual_is_zero, float* Q, uint32_t ldq,
                    float* P, uint32_t ldp, uint32_t r, uint32_t power_iters)
{
    if (!grad || !residual || !Q || !P) return ORACLE_EINVAL;
    if (m == 0 || n == 0 || r == 0 || r > m || r > n || ld < n || ldq < r || ldp < r ||
        power_iters == 0)
        return ORACLE_EINVAL;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_EINVAL;
    const int bf = (dtype == ORACLE_BF16);

    /* error feedback: D = G + E_old, kept in the residual buffer (fp32) */
    for (uint32_t i = 0; i < m; ++i)
        for (uint32_t j = 0; j < n; ++j) {
            float g = load_as_f32(grad, dtype, (uint64_t)i * ld + j);
            float e = residual_is_zero ? 0.0f : residual[(size_t)i * n + j];
            residual[(size_t)i * n + j] = g + e;
        }

    for (uint32_t it = 0; it < power_iters; ++it) {
        float* Qop = factor_operand(Q, n, ldq, r, bf);
        if (!Qop) return ORACLE_ENOMEM;
        contract_P(residual, m, n, Qop, r, bf, P, ldp);            /* P = D Q       */
        free(Qop);
        int rc = orthonormalise(P, m, r, ldp);                     /* P -> P^       */
        if (rc) return rc;
        float* Pop = factor_operand(P, m, ldp, r, bf);
        if (!Pop) return ORACLE_ENOMEM;
        contract_Q(residual, m, n, Pop, r, bf, Q, ldq);            /* Q = D^T P^    */
        free(Pop);
    }
    return ORACLE_OK;
}

/* The steps of oracle_compress one by one, for checks of a full-size run on sampled rows and
 * columns: the same routines the whole step calls, with the operand roundings of R10. */
int oracle_contract_p(const float* D, uint32_t m, uint32_t n, const float* Q, uint32_t ldq, uint32_t r,
                      int dtype, float* P, uint32_t ldp)
{
    if (!D || !Q || !P || m == 0 || n == 0 || r == 0 || ldq < r || ldp < r) return ORACLE_EINVAL;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_EINVAL;
    const int bf = (dtype == ORACLE_BF16);
    float* Qop = factor_operand(Q, n, ldq, r, bf);
    if (!Qop) return ORACLE_ENOMEM;
    contract_P(D, m, n, Qop, r, bf, P, ldp);
    free(Qop);
    return ORACLE_OK;
}

int oracle_contract_q(const float* D, uint32_t m, uint32_t n, const float* P, uint32_t ldp, uint32_t r,
                      int dtype, float* Q, uint32_t ldq)
{
    if (!D || !Q || !P || m == 0 || n == 0 || r == 0 || ldq < r || ldp < r) return ORACLE_EINVAL;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_EINVAL;
    const int bf = (dtype == ORACLE_BF16);
    float* Pop = factor_operand(P, m, ldp, r, bf);
    if (!Pop) return ORACLE_ENOMEM;
    contract_Q(D, m, n, Pop, r, bf, Q, ldq);
    free(Pop);
    return ORACLE_OK;
}

int oracle_orthonormalise(float* P, uint32_t m, uint32_t r, uint32_t ldp)
{
    if (!P || m == 0 || r == 0 || ldp < r) return ORACLE_EINVAL;
    return orthonormalise(P, m, r, ldp);
}

double oracle_reconstruct_one(const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                              uint32_t r, uint32_t i, uint32_t j, int dtype)
{
    const int bf = (dtype == ORACLE_BF16);
    double s = 0.0;
    for (uint32_t c = 0; c < r; ++c) {
        float p = P[(size_t)i * ldp + c], q = Q[(size_t)j * ldq + c];
        if (bf) { p = round_through_bf16(p); q = round_through_bf16(q); }
        s += (double)p * (double)q;
    }
    float m32 = (float)s;
    if (bf) m32 = round_through_bf16(m32);
    return (double)m32;
}

int oracle_decompress(const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                      uint32_t m, uint32_t n, uint32_t r, float* residual,
                      void* grad_out, int dtype, uint64_t ld)
{
    if (!P || !Q || !residual || !grad_out) return ORACLE_EINVAL;
    if (m == 0 || n == 0 || r == 0 || ld < n || ldq < r || ldp < r) return ORACLE_EINVAL;
    if (dtype != ORACLE_F32 && dtype != ORACLE_BF16) return ORACLE_EINVAL;
    #pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < (int64_t)m; ++i) {
        for (uint32_t j = 0; j < n; ++j) {
            /* M^[i,j] = sum_c P^[i,c] Q[j,c]; rounded to the gradient's dtype */
            float w = (float)oracle_reconstruct_one(P, ldp, Q, ldq, r, (uint32_t)i, j, dtype);
            if (dtype == ORACLE_BF16) ((uint16_t*)grad_out)[(size_t)i * ld + j] = oracle_f32_to_bf16(w);
            else                      ((float*)grad_out)[(size_t)i * ld + j] = w;
            /* E_new = D - M^ as transmitted */
            residual[(size_t)i * n + j] = residual[(size_t)i * n + j] - w;
        }
    }
    return ORACLE_OK;
}
