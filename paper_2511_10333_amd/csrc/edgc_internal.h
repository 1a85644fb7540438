// Internal declarations shared by the HIP translation units of libedgc.
// Nothing here is part of the public ABI (include/edgc.h is).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "edgc.h"

namespace edgc {

// Scratch owned by a context.  Sized once in edgc_create; hot calls only use it.
struct Scratch {
    // entropy
    float*              mm_part      = nullptr;  // [2 * kMaxReduceBlocks] per-block (lo, hi)
    unsigned int*       done_counter = nullptr;  // [4] last-block tickets and the overflow gate, zero between calls
    uint16_t*           part16       = nullptr;  // [part16_blocks][65536] 16-bit counters per block
    uint32_t            part16_blocks = 0;
    unsigned long long* wide         = nullptr;  // [65536] 64-bit credits per key, zero between calls
    unsigned long long* totals       = nullptr;  // [65536] counts per bf16 bit pattern
    unsigned long long* counts       = nullptr;  // [max_bins] histogram when the caller gives none
    void*               range        = nullptr;  // RangeParams
    void*               result_dev   = nullptr;  // edgc_entropy_result
    // compress / decompress
    float*  part      = nullptr;   // split-K partial factors [S][rows][rank_pad]
    size_t  part_elems = 0;
    double* gram_part = nullptr;   // [gram_blocks][rank_pad*rank_pad]
    size_t  gram_part_elems = 0;
    double* gram      = nullptr;   // [rank_pad*rank_pad]
    double* rinv      = nullptr;   // rinv_elems(max_rank): upper-triangle tiles of R^-1
    void*   pt        = nullptr;   // operand copy of P^ transposed: [planes][rank_pad][rows_pad] bf16
    size_t  pt_bytes  = 0;
};

constexpr int kMaxReduceBlocks = 4096;

// Doubles behind `rinv`: the upper-triangle 16x16 tiles of R^-1 for a rank padded to a multiple of 16
inline size_t rinv_elems(uint32_t max_rank)
{
    const size_t t = (static_cast<size_t>(max_rank) + 15) / 16;
    return t * (t + 1) / 2 * 256;
}

// Largest row count, column count or leading dimension of a compressed matrix: the kernels keep
// lane offsets of up to four rows (4 * leading dimension + column) in 32 bits.
constexpr uint64_t kMaxDim = 1ull << 28;

// ---------------------------------------------------------------------------
// Grouped launches of the compressor.  Every compressor kernel works on a list of tensors:
// the grid is the concatenation of the tensors' block ranges and a block finds its tensor
// from `first`.  The list travels by value in the kernel arguments (no table upload); a
// single-tensor call is a group of one.
// ---------------------------------------------------------------------------
constexpr int kMaxGroup = 16;

struct TensorArgs {
    const void* G;          // gradient (m x n, ldg), or null: D is re-read as it stands
    float*  E;              // residual: E_old in, D out (P-pass); D in, E_new out (decompress)
    float*  Q;              // n x r (ldq)
    float*  P;              // m x r (ldp)
    void*   out;            // decompressed gradient (m x n, ldo)
    float*  part;           // split partials: [S][rows][rank_pad]
    double* gram_part;      // per-block upper-triangle Gram tiles
    double* gram;           // summed Gram tiles
    double* rinv;           // inverse factor R^-1: upper-triangle 16x16 tiles, row-major over (tk <= tc)
    void*   pt;             // transposed bf16 copy of P^: [planes][rank_pad][m_pad]
    const double* tiles;    // what k_chol reads: gram_part (nb sets) or gram (one set)
    uint64_t ldg, ldo;
    uint32_t ldq, ldp, m, n, m_pad;
    int32_t  e_zero;
    uint32_t sp;            // column splits the P-pass wrote (k_reduce_gram sums them)
    uint32_t sq;            // row splits the Q-pass wrote (k_reduce_q sums them)
    uint32_t nb;            // Gram sets in `tiles`
    uint32_t d0, d1;        // decomposition of the launch at hand (set by the host before it)
    uint32_t first;         // first block of this tensor in the grouped grid
};

struct Group {
    uint32_t count;
    uint32_t r;             // rank, the same for every tensor of a group
    uint32_t stream;        // 1: the group's residual is too large to stay in the last-level cache:
                            //    the Q-pass reads D, and the P-pass E_old, with non-temporal loads.
                            //    0: both are ordinary loads, so that D is still cached when the
                            //    decompress reads it again and E_new when the next step's P-pass does
    uint32_t defer;         // 1: deferred subtraction: the residual buffer holds D between steps and the
                            //    next P-pass subtracts M^ = P^ Q^T itself; the decompress only writes M^
    TensorArgs t[kMaxGroup];
};

// scratch capacities behind one tensor's pointers (host side only)
struct TensorScratch {
    size_t part_elems = 0, gram_part_elems = 0;
};

// Scratch of one position of a batch (edgc_reserve_batch), sized for that position's shape.
struct BatchSlot {
    uint32_t rows = 0, cols = 0;
    float*  part = nullptr;
    double* gram_part = nullptr;
    double* gram = nullptr;
    double* rinv = nullptr;
    void*   pt = nullptr;
    TensorScratch cap;
};

// Kernel ids for the optional per-kernel event timing (edgc_profile_begin/end).
enum KernelId {
    KID_SET_RANGE = 0, KID_MINMAX, KID_HIST, KID_SAMPLE_IDX, KID_INIT_Q, KID_PASS_P,
    KID_REDUCE_GRAM, KID_GRAM_SUM, KID_CHOL, KID_APPLY, KID_PASS_Q, KID_REDUCE_Q, KID_DECOMPRESS,
    KID_PASS_P_DEFERRED, KID_WIDE_HIST, KID_WIDE_REDUCE, KID_COUNT
};
extern const char* const kKernelNames[KID_COUNT];

struct ProfRec {
    int kid;
    hipEvent_t a, b;
    double bytes, flops;
};

struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> pool;   // created in edgc_profile_begin, never in a hot call
    size_t next = 0;
    std::vector<ProfRec> recs;
    double empty_pair_ms = 0.0;     // elapsed time an empty event pair reports
};

}  // namespace edgc

struct edgc_ctx {
    int device = 0;
    uint32_t max_bins = 0, max_rank = 0;
    uint64_t max_rows = 0, max_cols = 0;
    int num_cu = 256;
    // launch-shape overrides for sweeps (blocks per CU aimed at by the P-pass, Q-pass and
    // decompress); 0 = the built-in choice
    uint32_t tune_p = 0, tune_q = 0, tune_d = 0;
    int tune_stream = -1;   // -1: by size; 0 / 1: force cached / non-temporal reads of D in the Q-pass
    int tune_dfull = -1;    // write-only decompress of whole-tile groups: -1 built-in choice (above rank
                            // 64 the whole-tile kernel, 8 waves per block); 0 the general kernel; 4 / 8
                            // the whole-tile kernel with that many waves per block at every rank
    int tune_full = -1;     // P-pass of whole-tile groups: -1 built-in choice; 0 the general kernels;
                            // 1 / 2 the whole-tile kernel with the Q rows requested early / late
    int tune_pwaves = -1;   // waves per block of that kernel: -1 built-in choice (8 above rank 64), 4 or 8
    int tune_qfull = -1;    // Q-pass of whole-tile groups: -1 built-in choice; 0 the general kernel; 4 / 8 the
                            // pipelined kernel with that many waves per block
    int tune_apply = -1;    // k_apply above rank 64: 4 = four waves (64 rows) per block, 8 = eight (128 rows)
    int tune_ept = 0;       // items per thread of the histogram of a small sample (the range pass takes twice as many)
    int tune_pattern = 1;   // entropy estimate: 1 one read into 16-bit counters per block where that applies
                            // (bf16 samples, fp32 on more than 16384 bins); 0 the plain kernels only; 3 as 1,
                            // and every such estimate reports a counter overflow (tests of the redo path)
    long long tune_pattern_min = 32 << 20;  // bf16 samples from this many elements on are counted by bit pattern
                                            // (on more than 16384 bins: from an eighth of it on)
    edgc::Scratch s;
    std::vector<edgc::BatchSlot> batch;
    edgc::Profiler prof;
    std::string last_error;
};

namespace edgc {

inline int fail(edgc_ctx* ctx, int code, const std::string& msg)
{
    if (ctx) ctx->last_error = msg;
    return code;
}

#define EDGC_HIP_TRY(ctx, expr)                                                              \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return ::edgc::fail((ctx), EDGC_EHIP,                                            \
                                std::string(#expr) + ": " + hipGetErrorString(e_));          \
    } while (0)

// Brackets one kernel launch with a pair of events when profiling is on.
struct ProfScope {
    edgc_ctx* ctx;
    hipStream_t st;
    hipEvent_t stop = nullptr;
    ProfScope(edgc_ctx* c, hipStream_t s, int kid, double bytes, double flops) : ctx(c), st(s)
    {
        Profiler& p = c->prof;
        if (!p.on || p.next + 2 > p.pool.size() || p.recs.size() == p.recs.capacity()) return;
        hipEvent_t a = p.pool[p.next++];
        stop = p.pool[p.next++];
        (void)hipEventRecord(a, st);
        p.recs.push_back(ProfRec{kid, a, stop, bytes, flops});
    }
    ~ProfScope() { if (stop) (void)hipEventRecord(stop, st); }
};
#define EDGC_LAUNCH(ctx, st, kid, bytes, flops, ...)                 \
    do {                                                             \
        ::edgc::ProfScope prof_scope_((ctx), (st), (kid), (bytes), (flops)); \
        __VA_ARGS__;                                                 \
    } while (0)

// splitmix64 output function on seed + golden * (ctr + 1); the sampler's slot and
// the seeded start of Q are drawn from it (host and device).
__host__ __device__ inline uint64_t mix64(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + 0x9E3779B97F4A7C15ull * (ctr + 1ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// Geometry of the chunk-strided sample (GDS, Sec. IV-B), computed on the host.
struct SampleGeom {
    uint64_t n;         // elements in the buffer
    uint64_t stride;    // chunk stride = 1 / beta
    uint64_t slot;      // sampled residue class of the chunk index
    uint64_t n_chunks;  // number of sampled chunks
    uint64_t n_items;   // n_chunks * ipc
    uint64_t n_sampled; // sampled elements
    uint32_t chunk;     // elements per chunk
    uint32_t ipc;       // items (vectors of VEC elements) per chunk
    uint32_t vec;       // elements per item: 1, 4 (fp32) or 8 (bf16)
};

// The buffers of one entropy estimate: the sample is the union of every buffer's own
// chunk-strided sample, and range, histogram and entropy are taken over that union.
constexpr int kMaxEntGroup = 32;
struct EntGroup {
    uint32_t count;
    uint32_t _pad;
    uint64_t n_items;       // over all buffers
    uint64_t n_sampled;     // over all buffers
    const void* base[kMaxEntGroup];
    SampleGeom geom[kMaxEntGroup];
};

SampleGeom make_geom(const void* base, edgc_dtype dt, uint64_t n, uint64_t stride, uint32_t chunk,
                     uint64_t seed, uint64_t step, bool allow_vec = true);

// launchers (entropy.hip)
int launch_entropy(edgc_ctx* ctx, const EntGroup& grp, edgc_dtype dt, uint32_t bins,
                   const float* range, edgc_entropy_result* out, uint64_t* counts_out, hipStream_t st);
int launch_sample_indices(edgc_ctx* ctx, const SampleGeom& g, uint64_t* idx, uint64_t cap,
                          hipStream_t st);
// the estimate on the file-scope scratch array (no allocation anywhere): at most kStaticMaxBins bins
constexpr uint32_t kStaticMaxBins = 65536;
int resolve_static_scratch(edgc_ctx* ctx);      // once per device, from edgc_create
int launch_entropy_static(edgc_ctx* ctx, const EntGroup& grp, edgc_dtype dt, uint32_t bins, const float* range,
                          edgc_entropy_result* out, uint64_t* counts_out, hipStream_t st);

// launchers (compress.hip)
int launch_init_q(edgc_ctx* ctx, float* Q, uint32_t n, uint32_t ldq, uint32_t c0, uint32_t c1,
                  uint64_t seed, hipStream_t st);
// `g` holds the tensors' pointers, shapes and scratch; the launchers fill in the rest.
// phase 0: whole step; 1: up to P = D Q (not orthonormalised); 2: orthonormalise P as it stands, Q-pass
int launch_compress(edgc_ctx* ctx, Group& g, const TensorScratch* cap, edgc_dtype dt,
                    uint32_t power_iters, hipStream_t st, int phase = 0);
int launch_decompress(edgc_ctx* ctx, Group& g, edgc_dtype dt, hipStream_t st);
int launch_copy_rows(edgc_ctx* ctx, const void* src, uint64_t ld_src, void* dst, uint64_t ld_dst,
                     uint32_t m, uint32_t n, uint32_t elem_bytes, hipStream_t st);
int prepare_compress_kernels(edgc_ctx* ctx);
int prepare_entropy_kernels(edgc_ctx* ctx);
size_t compress_part_elems(uint64_t max_rows, uint64_t max_cols, uint32_t max_rank, int num_cu);

// the P-pass of groups made of whole tiles only (pass_p_full.hip)
bool pass_p_full_applies(const Group& g, edgc_dtype dt, int rank_tiles, uint32_t waves);
hipError_t launch_pass_p_full(const Group& g, edgc_dtype dt, int rank_tiles, uint32_t blocks, bool qlate,
                              uint32_t waves, hipStream_t st);
hipError_t prepare_pass_p_full();
// the write-only reconstruction of groups made of whole tiles only (decompress_full.hip)
bool decompress_full_applies(const Group& g, edgc_dtype dt, uint32_t waves);
hipError_t launch_decompress_full(const Group& g, edgc_dtype dt, int rank_tiles, uint32_t blocks, uint32_t waves,
                                  hipStream_t st);
hipError_t prepare_decompress_full();
// pass_q_full.hip: the Q-pass of groups of whole tiles, the next stage's rows requested while the
// current stage is multiplied
bool pass_q_full_applies(const Group& g, edgc_dtype dt, int rank_tiles, uint32_t waves);
hipError_t launch_pass_q_full(const Group& g, edgc_dtype dt, int rank_tiles, uint32_t blocks, uint32_t waves,
                              hipStream_t st);

}  // namespace edgc
