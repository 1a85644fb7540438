/*
 * EDGC CPU oracle -- TEST INFRASTRUCTURE, NOT A PRODUCT PATH.
 *
 * A plain, slow, obviously-correct C implementation of what the EDGC
 * data-parallel hot path computes: down-sampled gradient entropy (GDS,
 * Sec. IV-B with Definition 1 / Eq. (1)), the entropy -> rank model (CQM:
 * Lemma 1, Theorem 1, Theorem 3 in the Appendix; Sec. IV-D-2 warm-up;
 * Algorithm 1 window-based adjustment with Constraint 2) and the rank-r
 * low-rank compressor with error feedback (Sec. II-B, Sec. III-B, Sec. VII).
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this library.  It shares no code, header, table or constant generator with
 * the HIP implementation.  Storage is fp32 where the method stores fp32;
 * every accumulation is fp64; no fusion and no reordering of any sum beyond
 * what the definitions state.  OpenMP only splits independent outputs: rows
 * of P and of M^, and, for Q = D^T P^, ranges of 64 columns of D per thread
 * (a loop interchange so that D is walked along its rows; every sum over
 * i = 0 .. m-1 still runs in that order, one term at a time).
 *
 * Readings of the paper where it is silent or ambiguous (each one is also
 * restated at the function that applies it):
 *   R1  Eq. (1) is estimated with an equal-width B-bin histogram of the
 *       sample; both the discrete Shannon entropy (bits) and the histogram
 *       estimate of the differential entropy (nats) = H*ln2 + ln(bin width)
 *       are returned.  Theorem 3 consumes the differential form.
 *   R2  The beta-subset (Sec. IV-B) is chunk-strided: element i is sampled
 *       iff ((i / chunk) mod stride) == slot, slot = mix64(seed, step) mod
 *       stride, stride = 1/beta.
 *   R3  Range = [min, max] of the finite sample (or a caller range);
 *       non-finite samples are counted and skipped; the bin index is computed
 *       in fp32 as trunc((x - lo) * (B / (hi - lo))) with separately rounded
 *       subtract, divide and multiply (no FMA), clamped to [0, B-1].
 *   R4  Lemma 1 is applied with m' = min(m,n), n' = max(m,n); Theorem 1's
 *       random draws are replaced by the mid-point quantiles (k - 1/2)/m'.
 *   R5  g^{-1}(t) = smallest integer r with g(r) <= t.
 *   R6  The reference point of Theorem 3 is anchored: H0 = mean entropy of
 *       the first window, r0 = r_ref (r_max unless the caller overrides it).
 *   R7  Algorithm 1 runs on an un-snapped integer state r_prev; the emitted
 *       rank is the smallest allowed value >= that state inside [r_min, r_max],
 *       or, when there is none, the largest allowed value inside the bounds
 *       (r_max of Sec. IV-D-1 is never exceeded); an allowed set with no
 *       member inside the bounds is an error, and so is r_min = 0.
 *   R8  The compressor is one (or more) warm-started subspace iteration
 *       steps: P = D Q, orthonormalise P, Q = D^T P, M^ = P Q^T with
 *       D = G + E_old, E_new = D - M^ (PowerSGD, the method the paper cites).
 *   R9  Orthonormalisation = QR's Q-factor with positive diagonal R, by
 *       modified Gram-Schmidt in fp64; a column whose remaining norm is below
 *       1e-30 * ||P||_F becomes zero.
 *   R10 With bf16 gradients the contraction operands (D, Q, P^) are rounded
 *       to bf16 (round-to-nearest-even) before each contraction, products are
 *       accumulated exactly (fp64 here); the output M^ is rounded to bf16 and
 *       E_new = D - widen(out) also absorbs that rounding.
 *
 * Pins (tests/test_oracle_*.py, no GPU): brute-force index enumeration,
 * H = 0 / log2 B / 1 bit special cases, NumPy fp32 brute-force bins,
 * Lemma 2 and the Laplace closed form, F(a)=0, F(b)=1, sum of quantiles =
 * m'n', SVD tails of seeded Gaussians (Theorem 1), hand tables for
 * Algorithm 1, exactly-rank-r reconstruction, P^T P = I, Pythagoras,
 * Eckart-Young bound, power-method convergence, error-feedback telescoping.
 */
#ifndef EDGC_ORACLE_H
#define EDGC_ORACLE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORACLE_F32 = 0, ORACLE_BF16 = 1 };
enum { ORACLE_OK = 0, ORACLE_EINVAL = -1, ORACLE_ENOMEM = -2, ORACLE_ENONFINITE = -5 };

typedef struct {
    double   H_bits;       /* discrete Shannon entropy of the histogram, log2        */
    double   h_diff_nats;  /* H_bits*ln2 + ln((hi-lo)/B); -inf when hi == lo          */
    float    lo, hi;       /* histogram range                                         */
    uint64_t n_sampled;    /* elements selected by the sampling predicate             */
    uint64_t n_nonfinite;  /* of those, NaN/Inf (skipped)                              */
} oracle_entropy_result;

typedef struct {
    uint32_t m, n;             /* reference matrix shape fed to g(r; m, n)            */
    uint32_t r_min, r_max;     /* rank bounds (Sec. IV-D-1)                           */
    uint32_t step_limit;       /* s of Constraint 2 (paper: 8)                        */
    const uint32_t* allowed;   /* optional ascending list of emit-able ranks          */
    uint32_t n_allowed;
    double   eta;              /* T_com(r) = eta * r; 0 => T_com = 0                  */
    uint64_t total_iters;      /* for the >= 10 % warm-up rule                        */
    double   min_warmup_frac;  /* paper: 0.10                                         */
    uint32_t r_ref;            /* r0 of Theorem 3; 0 => r_max (the paper's choice)    */
} oracle_rank_params;

typedef struct {
    int32_t  have_ref;
    int32_t  compressing;
    double   H_ref;
    double   r_prev;
    uint64_t iters_seen;
} oracle_rank_state;

typedef struct {
    uint32_t rank;          /* 0 => still warm-up (send uncompressed)                 */
    uint32_t _pad;
    double   r_unclamped;   /* r_new of Theorem 3 before step limit / clamp           */
    double   H_mean;
    double   T_com;
} oracle_rank_decision;

uint64_t oracle_mix64(uint64_t seed, uint64_t ctr);
uint64_t oracle_sample_slot(uint64_t seed, uint64_t step, uint64_t stride);
/* Writes the sampled element indices in increasing order; returns their number
 * (idx may be NULL to only count; at most cap entries are written). */
uint64_t oracle_sample_indices(uint64_t n, uint64_t stride, uint32_t chunk,
                               uint64_t seed, uint64_t step, uint64_t* idx, uint64_t cap);

int oracle_entropy(const void* grad, int dtype, uint64_t n, uint64_t stride, uint32_t chunk,
                   uint64_t seed, uint64_t step, uint32_t bins, const float* range_lo_hi,
                   oracle_entropy_result* out, uint64_t* counts);

double oracle_mp_cdf(double lambda, uint32_t m, uint32_t n);
double oracle_mp_quantile(double p, uint32_t m, uint32_t n);
/* g[r], r = 0..min(m,n): Theorem 1's error estimate.  Returns min(m,n). */
int64_t oracle_g_table(uint32_t m, uint32_t n, double* g);
int oracle_select_rank(oracle_rank_state* st, const double* H_window, uint32_t k,
                       uint64_t iters_in_window, const oracle_rank_params* prm,
                       oracle_rank_decision* out);

void oracle_init_q(float* Q, uint32_t n, uint32_t ldq, uint32_t col_begin, uint32_t col_end,
                   uint64_t seed);
int oracle_compress(const void* grad, int dtype, uint32_t m, uint32_t n, uint64_t ld,
                    float* residual, int residual_is_zero, float* Q, uint32_t ldq,
                    float* P, uint32_t ldp, uint32_t r, uint32_t power_iters);
int oracle_decompress(const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                      uint32_t m, uint32_t n, uint32_t r, float* residual,
                      void* grad_out, int dtype, uint64_t ld);
/* The steps of oracle_compress one by one (the routines the whole step is made of), so that a
 * full-size run can be checked on gathered rows and columns:
 *   oracle_contract_p      P = D Q       D: m x n dense (e.g. gathered rows of D), Q: n x r
 *   oracle_contract_q      Q = D^T P^    D: m x n dense (e.g. gathered columns of D), P: m x r
 *   oracle_orthonormalise  P -> P^ in place (R9)
 * dtype selects the operand rounding of R10 (ORACLE_BF16: D, Q, P^ rounded to bf16). */
int oracle_contract_p(const float* D, uint32_t m, uint32_t n, const float* Q, uint32_t ldq, uint32_t r,
                      int dtype, float* P, uint32_t ldp);
int oracle_contract_q(const float* D, uint32_t m, uint32_t n, const float* P, uint32_t ldp, uint32_t r,
                      int dtype, float* Q, uint32_t ldq);
int oracle_orthonormalise(float* P, uint32_t m, uint32_t r, uint32_t ldp);
/* One element of M^ = P^ Q^T (fp64 accumulate, then rounded as decompress does);
 * lets a test check sampled outputs of a full-size run one by one. */
double oracle_reconstruct_one(const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                              uint32_t r, uint32_t i, uint32_t j, int dtype);

float    oracle_bf16_to_f32(uint16_t h);
uint16_t oracle_f32_to_bf16(float x);
int      oracle_num_threads(void);
void     oracle_set_num_threads(int n);   /* threads for the loops over independent outputs */

#ifdef __cplusplus
}
#endif
#endif
