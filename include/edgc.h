/*
 * edgc.h -- C ABI of the MI355X (gfx950) implementation of EDGC's per-step
 * data-parallel hot path (EDGC: Entropy-driven Dynamic Gradient Compression,
 * arXiv 2511.10333):
 *
 *   1. down-sampled gradient-entropy estimation   (GDS, Sec. IV-B; Eq. (1))
 *   2. entropy window -> compression rank         (CQM, Theorem 3 with g of
 *      Theorem 1 / Lemma 1; warm-up Sec. IV-D-2; Algorithm 1, Constraint 2)
 *   3. rank-r low-rank compress / decompress with an error-feedback residual
 *      (Sec. II-B, Sec. III-B, Sec. VII; PowerSGD-style subspace iteration)
 *   4. rank bounds from measured compress / decompress times, the linear
 *      communication-time model and stage-aligned ranks (Sec. IV-D-1,
 *      Sec. IV-D-4, Algorithm 2), iteration sampling rate (Sec. IV-B)
 *   5. the same entropy estimate and compressor over all gradient tensors of
 *      a pipeline stage in one launch sequence (batched calls), with the
 *      error-feedback residual stored as E or kept as D plus the factors
 *      ("deferred"), and the compress as one call or in the two phases between
 *      which a data-parallel step exchanges P
 *
 * Conventions
 *   - Every function returns an edgc_status (0 = OK, < 0 = error).  No C++
 *     exception crosses this boundary.
 *   - "device" pointers are HIP device memory on the context's GPU, owned by
 *     the caller; "host" pointers are ordinary process memory.  The library
 *     allocates device memory only in edgc_create (scratch) and frees it in
 *     edgc_destroy (and, for batches, in edgc_reserve_batch).  Hot calls
 *     never allocate, never free and never
 *     synchronise the stream; they only enqueue work on `hip_stream`
 *     (a hipStream_t passed as void*, NULL = the default stream).
 *   - Matrices are row-major.  A gradient G is m x n with leading dimension
 *     ld (elements); the residual is dense m x n fp32; factors P (m x r) and
 *     Q (n x r) are fp32 with leading dimensions ldp, ldq >= r.
 *   - One context serves one stream at a time: calls that share a context
 *     share its scratch, so overlapping calls on the same context race.
 *   - Argument errors are reported before anything is launched.
 */
#ifndef EDGC_H
#define EDGC_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { EDGC_F32 = 0, EDGC_BF16 = 1 } edgc_dtype;

typedef enum {
    EDGC_OK         =  0,
    EDGC_EINVAL     = -1,   /* bad argument (null / misaligned pointer, size out of range)  */
    EDGC_ENOMEM     = -2,   /* allocation failed (edgc_create, edgc_reserve_batch)         */
    EDGC_EHIP       = -3,   /* a HIP call failed; see edgc_last_error                      */
    EDGC_ENOTIMPL   = -4,
    EDGC_ENONFINITE = -5    /* empty sample, or no finite value in it                      */
} edgc_status;

typedef struct edgc_ctx edgc_ctx;   /* opaque; owns only scratch memory */

/* Creates a context on GPU `hip_device` with scratch sized for histograms of
 * up to max_bins bins and matrices of up to max_rows x max_cols at rank
 * <= max_rank (max_rank <= 128; max_rows, max_cols <= 2^28, which also bounds
 * every leading dimension of a compressed matrix in the calls below: beyond it
 * they return EDGC_EINVAL).  Besides what these sizes ask for, the entropy
 * estimate keeps 128 KiB of 16-bit counters per compute unit (32 MiB on a GPU of
 * 256) and two 512 KiB counter arrays.  *out is NULL on failure. */
int edgc_create(edgc_ctx** out, int hip_device, uint32_t max_bins, uint32_t max_rank,
                uint64_t max_rows, uint64_t max_cols);
int edgc_destroy(edgc_ctx* ctx);
/* Message of the last failing call on this context (context-owned string). */
const char* edgc_last_error(const edgc_ctx* ctx);

/* Optional per-kernel timing for benchmarks (not part of the method).  Between
 * edgc_profile_begin and edgc_profile_end every kernel the context launches is
 * bracketed by a pair of HIP events on the stream it runs on; the event pool
 * (2 * max_launches events) is created in edgc_profile_begin, never in a hot
 * call, and launches beyond the pool go untimed (16 <= max_launches <= 2^20).
 * edgc_profile_end synchronises the device and returns, per kernel name, the
 * launch count, the summed duration (each bracket minus what an empty event
 * pair reads, event_overhead_ms, measured in edgc_profile_begin) and the summed
 * algorithmic bytes and flops of those launches.
 * `kernel` points to a static string.  *n_out is the number of kernels seen
 * (may exceed cap; only cap entries are written). */
typedef struct {
    const char* kernel;
    uint64_t    launches;
    double      total_ms;
    double      bytes;
    double      flops;
    double      event_overhead_ms;
} edgc_kernel_stat;
int edgc_profile_begin(edgc_ctx* ctx, uint32_t max_launches);
int edgc_profile_end(edgc_ctx* ctx, edgc_kernel_stat* out, uint32_t cap, uint32_t* n_out);

/* ------------------------------------------------------------------------
 * 1. Gradient entropy of a down-sampled buffer (GDS, Sec. IV-B: a subset of
 *    each iteration's gradient, chosen at gradient sampling rate beta;
 *    entropy as in Definition 1 / Eq. (1), estimated with an equal-width
 *    histogram).
 *
 *    Sample: element i of the flat buffer is taken iff
 *        ((i / chunk) mod stride) == slot,  slot = mix64(seed, step) mod stride,
 *    stride = 1/beta; mix64(s, c) is the splitmix64 output function applied to
 *    s + 0x9E3779B97F4A7C15 * (c + 1).
 *    Bins: B equal-width bins over [lo, hi] = range of the finite sample (or
 *    the caller's range); index = trunc((x - lo) * (B / (hi - lo))) computed in
 *    fp32 with separately rounded subtract / divide / multiply, clamped to
 *    [0, B-1]; hi == lo puts everything in bin 0.  NaN/Inf are skipped and
 *    counted.
 * ------------------------------------------------------------------------ */
typedef struct {
    double   H_bits;        /* -sum p_i log2 p_i over the B bins                          */
    double   h_diff_nats;   /* H_bits*ln2 + ln((hi-lo)/B): histogram estimate of Eq. (1); */
                            /* this is what Theorem 3 consumes; -inf when hi == lo        */
    float    lo, hi;
    uint64_t n_sampled;     /* elements selected by the predicate                         */
    uint64_t n_nonfinite;   /* of those, skipped as NaN/Inf                               */
    int32_t  status;        /* EDGC_OK, or EDGC_ENONFINITE when no finite sample existed  */
    int32_t  _pad;
} edgc_entropy_result;

/* grad: device, n_elems of dtype.  range_lo_hi_or_null: host float[2] or NULL.
 * out: host, valid once the stream has been synchronised.  Pinned (device-
 * accessible, 8-byte aligned) memory is written by the kernel itself; any
 * other host memory by a device-to-host copy on `hip_stream`, which makes the
 * call wait for the stream.  counts_out_or_null: device, `bins` uint64 counters.
 * Errors: EDGC_EINVAL for null ctx/grad/out, stride == 0, chunk == 0,
 * bins == 0 or > max_bins, lo > hi; EDGC_ENONFINITE when the predicate selects
 * no element (known on the host).  A sample with no finite value is reported
 * in out->status. */
int edgc_entropy_estimate(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint64_t n_elems,
                          uint64_t stride, uint32_t chunk, uint64_t seed, uint64_t step,
                          uint32_t bins, const float* range_lo_hi_or_null,
                          edgc_entropy_result* out, uint64_t* counts_out_or_null,
                          void* hip_stream);

/* Writes the sampled element indices, ascending, to idx_out (device, capacity
 * `cap` entries) and their number to *n_out (host, known without the GPU).
 * Same predicate as edgc_entropy_estimate. */
int edgc_sample_indices(edgc_ctx* ctx, uint64_t n_elems, uint64_t stride, uint32_t chunk,
                        uint64_t seed, uint64_t step, uint64_t* idx_out, uint64_t cap,
                        uint64_t* n_out, void* hip_stream);

/* ------------------------------------------------------------------------
 * 2. Window of entropies -> rank.  Pure host code, deterministic, no GPU.
 *    H_mean = mean of the window (Sec. IV-D-3).  The first call stores it as
 *    the reference H_ref and returns rank 0.  Later calls evaluate Theorem 3
 *        r_new = g^{-1}( exp(H_ref - H_mean) * g(r_ref) ),
 *    g(r; m, n) = sqrt(sum of the min(m,n)-r smallest mid-point quantiles of
 *    the Marchenko-Pastur law of Lemma 1) (Theorem 1), g^{-1}(t) = smallest r
 *    with g(r) <= t.  Warm-up (Sec. IV-D-2): rank 0 until r_new < r_max and
 *    iters_seen >= min_warmup_frac * total_iters; compression then starts from
 *    r_prev = r_ref.  Algorithm 1: move r_prev towards r_new by at most
 *    step_limit (Constraint 2), clamp to [r_min, r_max], emit the smallest
 *    allowed rank >= r_prev inside [r_min, r_max], or the largest allowed
 *    rank inside the bounds when there is none (r_prev itself when no set is
 *    given), and T_com = eta * rank.  The emitted rank never leaves the
 *    bounds.  Entropies are the h_diff_nats values above.
 * ------------------------------------------------------------------------ */
typedef struct {
    uint32_t m, n;              /* reference matrix shape for g(r; m, n)                  */
    uint32_t r_min, r_max;      /* rank bounds, 1 <= r_min <= r_max <= min(m, n)          */
    uint32_t step_limit;        /* s of Constraint 2 (paper: 8)                           */
    const uint32_t* allowed;    /* host, ascending, or NULL                               */
    uint32_t n_allowed;
    double   eta;               /* T_com(r) = eta * r (Sec. IV-D-1); 0 => T_com = 0       */
    uint64_t total_iters;
    double   min_warmup_frac;   /* paper: 0.10                                            */
    uint32_t r_ref;             /* r0 of Theorem 3; 0 => r_max (the paper's choice)       */
} edgc_rank_params;

typedef struct {                /* caller-owned plain data; zero-initialise before use    */
    int32_t  have_ref;
    int32_t  compressing;
    double   H_ref;
    double   r_prev;            /* un-snapped state of Algorithm 1                        */
    uint64_t iters_seen;
} edgc_rank_state;

typedef struct {
    uint32_t rank;              /* 0 => warm-up: send uncompressed                        */
    uint32_t _pad;
    double   r_unclamped;       /* r_new before step limit and clamp                      */
    double   H_mean;
    double   T_com;
} edgc_rank_decision;

/* Errors: EDGC_EINVAL for null pointers, k == 0, bounds that are not
 * 1 <= r_min <= r_max <= min(m, n), a non-ascending allowed set or one with no
 * member inside [r_min, r_max]; EDGC_ENONFINITE for a NaN/Inf entropy. */
int edgc_select_rank(edgc_rank_state* state, const double* H_window, uint32_t k,
                     uint64_t iters_in_window, const edgc_rank_params* params,
                     edgc_rank_decision* out);

/* ------------------------------------------------------------------------
 * 3. Rank-r compressor with error feedback (Sec. II-B: power iteration and
 *    orthogonalisation give the low-rank factors; Sec. III-B / VII: error
 *    feedback).  One call of edgc_compress does, power_iters times,
 *        D = G + E_old (first iteration only; D replaces E_old in `residual`)
 *        P = D Q;  P <- orthonormal columns (QR Q-factor, positive diagonal R)
 *        Q = D^T P
 *    and edgc_decompress does  M^ = P Q^T -> grad_out,  E_new = D - M^ in
 *    `residual`.  With EDGC_BF16 the gradient and grad_out are bf16, the
 *    contraction operands are rounded to bf16 (nearest-even) and accumulated
 *    in fp32, and E_new = D - widen(bf16(M^)).  With EDGC_F32 operands are
 *    split into two bf16 planes (three MFMAs per product, ~2^-17 relative).
 * ------------------------------------------------------------------------ */

/* Fills columns [col_begin, col_end) of Q (device, n x ldq fp32) with seeded
 * N(0,1): element (j, c) is a pure function of (seed, j, c) -- Box-Muller on
 * two 53-bit uniforms from mix64(seed, 2k), mix64(seed, 2k+1), k = j*2^32 + c. */
int edgc_init_q(edgc_ctx* ctx, float* Q, uint32_t n, uint32_t ldq, uint32_t col_begin,
                uint32_t col_end, uint64_t seed, void* hip_stream);

/* grad: device m x n (ld) of dtype.  residual: device m x n fp32, in: E_old
 * (ignored when residual_is_zero != 0), out: D.  Q: device n x r (ldq), in:
 * warm start, out: D^T P.  P: device m x r (ldp), out: orthonormal columns.
 * Errors: EDGC_EINVAL for null pointers, r == 0, r > min(m, n), r > max_rank,
 * m > max_rows, n > max_cols, ld < n, ldp/ldq < r, power_iters == 0, or P/Q
 * not 16-byte aligned with ldp/ldq multiples of 4.
 * A column of P that is numerically dependent on the previous ones (its Cholesky
 * pivot not above 1e-11 times the column's squared norm, i.e. the pivot of the
 * Gram matrix scaled to a unit diagonal not above 1e-11) is set to zero. */
int edgc_compress(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint32_t m, uint32_t n,
                  uint64_t ld, float* residual, int residual_is_zero, float* Q, uint32_t ldq,
                  float* P, uint32_t ldp, uint32_t r, uint32_t power_iters, void* hip_stream);

/* residual: in D, out E_new.  grad_out: device m x n (ld) of dtype; may alias
 * the gradient passed to edgc_compress. */
int edgc_decompress(edgc_ctx* ctx, const float* P, uint32_t ldp, const float* Q, uint32_t ldq,
                    uint32_t m, uint32_t n, uint32_t r, float* residual, void* grad_out,
                    edgc_dtype dtype, uint64_t ld, void* hip_stream);

/* ------------------------------------------------------------------------
 * 4. Rank bounds, the linear communication-time model and stage alignment
 *    (host only, except edgc_measure_rank_costs which times this library's
 *    own kernels).
 *
 *    Sec. IV-D-1: compression at rank r pays when
 *        T_com(r) = T_compress + D_compressed / B + T_decompress <= D_original / B,
 *    the first rank that violates this closes the range and gives r_max; the
 *    footnote puts r_min between r_max/6 and r_max/4.  The same section models
 *    T_com(r) = eta * r.  Sec. IV-D-4 / Algorithm 2: stage i of the pipeline
 *    gets the rank whose predicted time is T_com(stage 1) + (i-1) * T_microBack,
 *    clamped to the bounds.  Sec. IV-B: with iteration sampling rate alpha the
 *    entropy is measured once every 1/alpha iterations of a window.
 * ------------------------------------------------------------------------ */
typedef struct {
    uint32_t rank;
    uint32_t _pad;
    double   t_compress;        /* seconds                                               */
    double   t_decompress;      /* seconds                                               */
    double   bytes_compressed;  /* D_compressed: what a rank-r exchange sends, in bytes  */
} edgc_rank_cost;

typedef struct {
    uint32_t r_max;             /* 0 => no candidate pays at this bandwidth              */
    uint32_t r_min;             /* ceil(r_max / divisor), at least 1; 0 when r_max == 0  */
    double   t_uncompressed;    /* D_original / B, seconds                               */
} edgc_rank_bounds_result;

/* costs: host, n entries in strictly ascending rank.  bandwidth in bytes per
 * second.  r_min_divisor in [4, 6].  t_com_out: host, n entries or NULL,
 * receives T_com of every candidate.  Candidates are scanned upwards and the
 * scan stops at the first one that violates the inequality, so a candidate
 * above it never becomes r_max even if it satisfies the inequality again.
 * Errors: EDGC_EINVAL for null pointers, n == 0, non-ascending ranks, a
 * non-positive bandwidth or size, a negative time, or a divisor outside
 * [4, 6]; EDGC_ENONFINITE for a NaN/Inf input. */
int edgc_rank_bounds(const edgc_rank_cost* costs, uint32_t n, double bytes_original,
                     double bandwidth, double r_min_divisor, edgc_rank_bounds_result* out,
                     double* t_com_out);

/* Least-squares fit through the origin of T_com(r) = eta * r over n points
 * (host arrays): eta = sum(r T) / sum(r^2); *mape_percent (may be NULL) =
 * 100 * mean(|T - eta r| / T).  Errors: EDGC_EINVAL for null pointers, n == 0,
 * a zero rank or a non-positive time; EDGC_ENONFINITE for NaN/Inf. */
int edgc_fit_eta(const uint32_t* ranks, const double* t_com, uint32_t n, double* eta,
                 double* mape_percent);

/* Algorithm 2.  ranks_out[0] = r_stage1 (stage 1 keeps the rank Algorithm 1
 * gave it); for stage i = 2..n_stages the budget is eta * r_stage1 +
 * (i-1) * t_microback and the rank is floor(budget / eta + 1e-9), clamped to
 * [r_min, r_max], then lowered to the largest allowed rank not above it (the
 * smallest allowed rank when none is; allowed: host, ascending, or NULL).
 * t_com_out (host, n_stages entries or NULL) receives eta * rank per stage.
 * Errors: EDGC_EINVAL for null ranks_out, n_stages == 0, eta <= 0,
 * t_microback < 0, r_min == 0, r_min > r_max or a non-ascending allowed set;
 * EDGC_ENONFINITE for NaN/Inf. */
int edgc_stage_ranks(uint32_t r_stage1, double t_microback, double eta, uint32_t r_min,
                     uint32_t r_max, const uint32_t* allowed, uint32_t n_allowed,
                     uint32_t n_stages, uint32_t* ranks_out, double* t_com_out);

/* Returns 1 when the entropy is to be measured at window-relative iteration
 * iter_in_window with period = 1/alpha (iterations 0, period, 2*period, ...),
 * 0 when not, EDGC_EINVAL when period == 0. */
int edgc_entropy_due(uint64_t iter_in_window, uint32_t period);

/* Times edgc_compress and edgc_decompress of this library on the caller's
 * buffers (arguments as for those two calls; grad_out must not alias grad
 * here) at each of n_ranks candidate ranks (host array, ascending): one
 * untimed round, then `reps` rounds of compress followed by decompress, each
 * call bracketed by HIP events on hip_stream.  costs_out[i] (host) receives
 * the rank, the mean time of either call in seconds, and bytes_compressed =
 * (m + n) * rank * 4 (P and Q in fp32, what the two exchanges of a data-
 * parallel step would carry).  deferred = 1 times the deferred form of the
 * residual instead (section 5: the timed compress subtracts P Q^T of the round
 * before on the way, the decompress only writes grad_out), which is what a
 * caller of the batched calls with deferred = 1 runs.  Overwrites residual, Q,
 * P and grad_out; synchronises the stream; not a hot-path call.
 * Errors: those of edgc_compress / edgc_decompress, EDGC_EINVAL for reps == 0,
 * n_ranks == 0 or deferred not 0 or 1. */
int edgc_measure_rank_costs(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint32_t m,
                            uint32_t n, uint64_t ld, float* residual, float* Q, uint32_t ldq,
                            float* P, uint32_t ldp, void* grad_out, const uint32_t* ranks,
                            uint32_t n_ranks, uint32_t reps, int deferred,
                            edgc_rank_cost* costs_out, void* hip_stream);

/* Measured ceilings of the device, for reading a kernel's throughput against:
 * what a plain streaming copy, a plain streaming read and a plain streaming
 * write of `bytes` reach (the passes of section 3 are bounded by HBM), and what a register-resident loop of
 * the 32x32x16 bf16 MFMA that the passes issue reaches.  Not part of the method
 * and not a hot-path call.
 *
 * buf_a, buf_b: two distinct device buffers of `bytes` each (16-byte aligned,
 * bytes a multiple of 16 and at least 8 * compute units * 1 KiB); buf_a is only
 * read (its contents do not matter but should be initialised), buf_b is
 * overwritten.  Each of the four kernels runs once untimed and then reps
 * times between a pair of events; synchronises the stream.
 * Errors: EDGC_EINVAL for null or misaligned arguments, equal buffers, a size
 * below the minimum or reps == 0; EDGC_EHIP for a failed HIP call. */
typedef struct {
    double   copy_gbs;          /* (bytes read + bytes written) / time, 1e9 bytes per second */
    double   read_gbs;          /* bytes read / time                                         */
    double   mfma_bf16_tflops;  /* dense bf16 MFMA, fp32 accumulate, 1e12 flop per second    */
    uint64_t bytes;             /* the size the memory figures were taken on                 */
    double   write_gbs;         /* bytes written / time (a plain fill of buf_b)              */
} edgc_device_peaks;

int edgc_measure_device_peaks(edgc_ctx* ctx, void* buf_a, void* buf_b, uint64_t bytes,
                              uint32_t reps, edgc_device_peaks* out, void* hip_stream);

/* ------------------------------------------------------------------------
 * 5. Batched calls: every gradient tensor of a pipeline stage in one launch
 *    sequence (Sec. IV-C: the rank is adjusted per window and per stage, so a
 *    stage's tensors share one rank; Sec. IV-D: DAC works on stages).  Each
 *    kernel of the compressor runs once over the whole list (the grid is the
 *    concatenation of the tensors' tiles), which removes the per-tensor launch
 *    and ramp-up cost that dominates for small matrices.
 *
 *    A tensor that compression cannot shrink is sent as it stands: one with a
 *    single row or column (biases, norm weights), or one whose factors are not
 *    smaller than itself, (m + n) r >= m n.  edgc_tensor_bypassed tells which
 *    (1 = sent as it stands, 0 = compressed, EDGC_EINVAL for a zero argument).
 *    For such a tensor edgc_compress_batch does nothing and
 *    edgc_decompress_batch copies grad to grad_out when the two differ; its
 *    residual, Q and P may be NULL.
 * ------------------------------------------------------------------------ */
typedef struct {
    const void* grad;           /* device m x n (ld) of the batch's dtype                  */
    void*       grad_out;       /* device m x n (ld_out); may be the same buffer as grad   */
    float*      residual;       /* device m x n fp32 (dense): as for edgc_compress         */
    float*      Q;              /* device n x ldq fp32                                     */
    float*      P;              /* device m x ldp fp32                                     */
    uint64_t    ld, ld_out;
    uint32_t    m, n, ldq, ldp;
    int32_t     residual_is_zero;
    uint32_t    deferred;       /* 0 or 1, the same for every tensor of a call: see below  */
} edgc_tensor;

int edgc_tensor_bypassed(uint32_t m, uint32_t n, uint32_t r);

/* Allocates the scratch of a batch: position i of later batch calls may hold a
 * tensor of up to rows[i] x cols[i] (host arrays).  Replaces an earlier
 * reservation; synchronises the device; not a hot call.  Like the context's
 * own scratch, the slots serve one stream at a time.
 * Errors: EDGC_EINVAL for null arrays, EDGC_ENOMEM. */
int edgc_reserve_batch(edgc_ctx* ctx, const uint32_t* rows, const uint32_t* cols, uint32_t count);

/* tensors: host array of `count` descriptors (read during the call only; the
 * device buffers they name are caller-owned).  Tensor i uses batch slot i.
 * What is computed per compressed tensor is exactly edgc_compress /
 * edgc_decompress at rank r; results are bit-identical to the single-tensor
 * calls when the launch shapes agree and equal to rounding otherwise.
 * edgc_compress_batch reads grad, ld, residual, residual_is_zero, Q, P;
 * edgc_decompress_batch reads P, Q, residual, grad_out, ld_out (and grad, ld
 * of tensors sent as they stand).
 * Errors: as for the single-tensor calls, EDGC_EINVAL also for count above the
 * reservation, a tensor larger than its slot, or descriptors that disagree in
 * `deferred`.  Nothing is launched when a descriptor is rejected.
 *
 * Deferred subtraction (deferred = 1).  The error feedback of Sec. III-B / VII
 * is E_t = D_t - M^_t with D_t = G_t + E_(t-1).  With deferred = 0 the
 * residual buffer holds E_t between steps, as for the single-tensor calls.
 * With deferred = 1 it holds D_t and E_t stays in factored form: the P and Q
 * buffers, which after the step hold P^_t and Q_t, stand in for M^_t.
 *   edgc_decompress_batch, deferred = 1: writes grad_out only; the residual
 *     buffer is neither read nor written and keeps D_t.
 *   edgc_compress_batch, deferred = 1: the residual buffer holds D_(t-1) and
 *     P, Q the factors of that step (unless residual_is_zero); the call forms
 *     D_t = G_t + D_(t-1) - P^_(t-1) Q_(t-1)^T on the way, M^_(t-1) computed
 *     and rounded exactly as the decompress wrote it, so the results equal
 *     the deferred = 0 chain bit for bit where the launch shapes agree.
 * This saves one read and one write of the fp32 residual per step.  The flag
 * of a compress call says what the buffer holds on entry, that of a
 * decompress call what it holds on return, so a chain may change over: after
 * decompress with 1, compress with 1; after decompress with 0 (or
 * edgc_residual_materialize_batch), compress with 0.  Between a deferred
 * decompress and the next compress the caller leaves P and Q untouched and
 * keeps r and dtype; before anything else that needs E_t itself (another
 * rank, a checkpoint of the residual, the single-tensor calls)
 * edgc_residual_materialize_batch carries the subtraction out:
 * residual <- residual - round_dtype(P Q^T).  With power_iters > 1 the
 * subtraction is part of the first iteration.  Tensors sent as they stand
 * ignore the flag. */
int edgc_compress_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count, edgc_dtype dtype,
                        uint32_t r, uint32_t power_iters, void* hip_stream);
int edgc_decompress_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                          edgc_dtype dtype, uint32_t r, void* hip_stream);
/* The compress in two phases, for a data-parallel step that exchanges the factors between them
 * (PowerSGD's two all-reduces, Sec. II-B; the inequality of Sec. IV-D-1 prices exactly these
 * two messages):
 *   edgc_compress_p_batch: error-feedback add and P-pass.  residual <- D, P <- D Q, NOT
 *     orthonormalised (what the ranks average).  Reads what edgc_compress_batch reads.
 *   edgc_compress_q_batch: orthonormalises P as it stands in the caller's buffer, then the
 *     Q-pass: P <- P^, Q <- D^T P^ (what the ranks average next).  Reads residual (D), P; grad,
 *     residual_is_zero and deferred are ignored.
 * The first followed by the second, with P untouched in between, is edgc_compress_batch with
 * power_iters = 1, bit for bit.  With deferred = 1 the caller stores the averaged Q back before
 * the decompress, so that the buffers hold the factors the reconstruction was formed from.
 * Errors: as for edgc_compress_batch. */
int edgc_compress_p_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count, edgc_dtype dtype,
                          uint32_t r, void* hip_stream);
int edgc_compress_q_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count, edgc_dtype dtype,
                          uint32_t r, void* hip_stream);
/* reads residual, P, Q of every compressed tensor; writes residual; `deferred` and the gradient
 * pointers of the descriptors are ignored.  r and dtype: those of the step that left P and Q. */
int edgc_residual_materialize_batch(edgc_ctx* ctx, const edgc_tensor* tensors, uint32_t count,
                                    edgc_dtype dtype, uint32_t r, void* hip_stream);

/* The entropy of a pipeline stage whose gradients are separate buffers (Sec.
 * IV-C / Algorithm 1 work with one entropy per stage): `count` (1..32)
 * buffers, grads[i] (host array of device pointers) of n_elems[i] elements
 * each.  Every buffer is sampled by its own element index with the same
 * (stride, chunk, seed, step), hence the same slot; the range, the histogram
 * and the entropy are taken over the union of those samples, and n_sampled /
 * n_nonfinite count over all buffers.  Other arguments, result and errors as
 * for edgc_entropy_estimate, which is this call with count = 1. */
int edgc_entropy_estimate_batch(edgc_ctx* ctx, const void* const* grads, const uint64_t* n_elems,
                                uint32_t count, edgc_dtype dtype, uint64_t stride, uint32_t chunk,
                                uint64_t seed, uint64_t step, uint32_t bins,
                                const float* range_lo_hi_or_null, edgc_entropy_result* out,
                                uint64_t* counts_out_or_null, void* hip_stream);

/* edgc_entropy_estimate for callers that cannot allocate device memory and cannot have a
 * library do it for them: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, result and errors as edgc_entropy_estimate, same kernels;
 * what differs is where the estimate's scratch lives (per-block ranges, last-block tickets,
 * the range parameters, the 64-bit histogram when counts_out_or_null is NULL, the result
 * before it is copied to non-pinned `out`): not in memory the context allocated but in a
 * file-scope device array of the library, 545 KiB, which every GPU the library runs on holds
 * from the load of the library's code to the end of the process.  Limit: bins <= 65536
 * (EDGC_EINVAL beyond, whatever max_bins the context was created with).  The call itself
 * allocates and frees nothing (no hipMalloc, no hipFree); the array's address on the context's
 * device is looked up once, in edgc_create.  All calls on one GPU, from whatever context or
 * stream, share that GPU's array: calls that overlap on one GPU race; calls in sequence are
 * safe (each call resets what must start at zero). */
int edgc_entropy_estimate_noalloc(edgc_ctx* ctx, const void* grad, edgc_dtype dtype, uint64_t n_elems,
                                  uint64_t stride, uint32_t chunk, uint64_t seed, uint64_t step,
                                  uint32_t bins, const float* range_lo_hi_or_null,
                                  edgc_entropy_result* out, uint64_t* counts_out_or_null,
                                  void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EDGC_H */
