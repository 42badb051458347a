// Internal declarations shared by the kernels and the host driver of libscd (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scd.h"
#include "scd_probe.h"

namespace scd {

constexpr int kWave = 64;        // gfx950 wavefront
constexpr int kBlock = 256;      // threads per workgroup of the row-pass and reduce kernels
constexpr int kWavesPerBlock = kBlock / kWave;
constexpr int kMaxRowsPerWg = 2048;

// What the next row pass over the remainder has to do; decided on the device by every workgroup
// from the same data, so that no launch depends on the host.
enum PassMode : int32_t {
    PASS_START = 0,  // first alternation of a term on an unchanged remainder (also computes ||R||^2)
    PASS_CONT = 1,   // a further alternation (Algorithm 4 lines 5-7)
    PASS_UPDATE = 2  // the term converged: subtract it (Algorithm 5 line 10), then act as PASS_START
};

// Device-resident position of the greedy loop.  `cur` is read by the level-0 row pass, which
// writes `next`; every later kernel of the sweep reads `next`; the last reduce copies next->cur.
struct State {
    int64_t k;         // terms completed
    int64_t w_target;  // stop once k == w_target
    int64_t passes;    // level-0 row passes executed
    int64_t updates;   // rank-1 updates executed
    double c_prev;     // c of the previous alternation of the current term (-inf before the first)
    double c_last;     // most recent c
    int32_t j;         // alternations completed for the current term (0: none yet)
    int32_t done;      // k == w_target and the remainder is up to date
    int32_t t0_given;  // the start of the current term is in the sign buffers, not the random stream
    int32_t warn;      // some term ended on max_iters
    int32_t norm_pending;  // the pass of this sweep summed squares: the last reduce records ||R_k||_F
    int32_t sweep_rng;     // levels >= 1 of this sweep read the random Kronecker signs
    int32_t active;        // written by the level-0 pass only: 0 = this sweep is skipped
    int32_t max_iters;
};

struct RowPassArgs {
    void* X;               // rows x cols, row-major.  level 0: the remainder (dtype), else f64 partial contraction
    int64_t rows, cols;
    int32_t level;
    int32_t rows_per_wg;
    const uint64_t* sign_cur;  // cols bits: Kronecker product of the current signs of the later modes
    const uint64_t* sign_rng;  // cols bits: the same for the random start of the next term
    const uint64_t* row_bits;  // rows bits: current signs of this level's mode
    void* partials;            // [grid][cols], element type of X
    double* u;                 // [rows]
    double* fparts;            // [grid] partial sums of squares (level 0)
    const double* cparts;      // partial sums of |v| written by the last reduce of the previous sweep
    int32_t ncparts;
    int32_t order;
    State* cur;
    State* next;
    void* c_out;               // [w] dtype
    int32_t* iters_out;        // [w]
    double total;              // prod dims (the mn of Algorithm 5 line 10)
    uint64_t* out_signs[SCD_MAX_ORDER];        // term-major outputs
    const uint64_t* cur_signs[SCD_MAX_ORDER];  // current sign bitsets per mode
    int32_t words[SCD_MAX_ORDER];
};

struct ReduceArgs {
    const void* partials;  // [nparts][cols]
    int32_t nparts;
    int32_t level;
    int64_t cols;
    int64_t rows;          // rows of this level (length of u)
    double* W;             // [cols] f64 sums
    const double* u;       // [rows]
    uint64_t* row_bits;    // rows bits <- sgn(u)
    int32_t final;         // last level: W is R^T s (the last mode's vector)
    uint64_t* last_bits;   // cols bits <- sgn(W)            (final)
    double* cparts;        // [ceil(cols/64)] sums of |W|    (final)
    uint64_t* rng_last;    // cols bits: random start of term k+1, last mode (final)
    const double* fparts;  // level-0 partial sums of squares
    int32_t nfparts;
    int32_t last_mode;
    double* trace;         // [w+1]
    uint64_t seed;
    State* cur;
    State* next;
};

struct KronArgs {
    int32_t order;
    int32_t term_offset;   // random signs are drawn for term cur->k + term_offset
    int32_t force;         // run even when the sweep is inactive (host-driven set-up)
    int32_t with_last;     // also write the last mode's random bitset
    int64_t dims[SCD_MAX_ORDER];
    const uint64_t* cur_signs[SCD_MAX_ORDER];
    uint64_t* kron_cur[SCD_MAX_ORDER];  // levels 0..order-3
    uint64_t* kron_rng[SCD_MAX_ORDER];  // levels 0..order-3
    uint64_t* rng_last;
    int64_t cols[SCD_MAX_ORDER];        // cols of level l = prod dims[l+1..]
    uint64_t seed;
    const State* cur;
    const State* next;
};

// Register-resident engine (scd_resident.hip): the whole remainder lives in the register files of a
// 16 x 16 grid of co-resident workgroups for as many terms as requested.
constexpr int kResGrid = 16;                       // workgroups per side
constexpr int kResThreads = 512;
constexpr int kResSlotWords = 512 + 8;             // exchange slot: up to 512 values + piggybacked scalars

struct ResidentResult {
    int64_t k;             // terms complete on exit
    int64_t alternations;  // row phases executed
    int64_t updates;
    uint32_t seq_u, seq_v; // last exchange sequence numbers used
    int32_t err;           // 1: a bounded wait ran out
    int32_t warn;          // a term ended on max_iters
    int64_t spins;         // re-reads of stale exchange data by thread 0 of workgroup 0 (diagnostic)
    int64_t flips;         // sparse engine: column signs that changed (each costs one column of R)
    int64_t flips_rows;    // sparse engine: row signs that changed (each costs one row of R)
    int64_t ticks[6];      // sparse engine, profile mode: 100 MHz ticks of workgroup 0 per phase
};

struct ResidentArgs {
    float* R;
    int64_t m, n;
    uint64_t seed;
    int64_t k_start, w_target;
    int32_t max_iters, max_spin;
    int32_t poll_delay;      // s_sleep units between publishing and the first read of the neighbours' data
    uint32_t seq_u, seq_v;   // sequence numbers already used by earlier launches
    uint64_t* xbuf;          // [2 kinds][2 parities][256 workgroups][kResSlotWords]
    uint64_t* S;
    uint64_t* T;
    float* c;
    int32_t* iters;
    double* trace;
    int32_t mw, nw;
    ResidentResult* res;
};

bool resident_supported(scd_dtype dt, int order, const int64_t* dims);
int resident_workgroups(const int64_t* dims);  // workgroups of the launch for a supported shape
hipError_t launch_resident(const ResidentArgs& a, hipStream_t st);

// Sparse engine (scd_sparse.hip): cached products updated from the flipped signs only; keeps R and its
// transpose in HBM.
constexpr int kSpGrid = 256;  // most workgroups of the persistent launch

struct SparseArgs {
    void* R;                 // m x n
    void* RT;                // n x m, the transpose, kept in step with R
    int64_t m, n;
    uint64_t seed;
    int64_t k_start, w_target;
    int32_t max_iters, max_spin;
    int32_t poll_delay;
    uint32_t seq;            // exchange sequence numbers already used
    uint64_t* xbuf;          // sparse_xbuf_bytes()
    uint64_t* S;
    uint64_t* T;
    void* c;
    int32_t* iters;
    double* trace;
    int32_t mw, nw;
    int32_t rs, cs;          // rows / columns owned per workgroup (multiples of 8)
    int32_t grid;            // workgroups of this launch (at most kSpGrid)
    int32_t profile;         // 1: workgroup 0 times its phases
    int32_t delay_width;     // > 0: finished terms wait in a list of this length before they are subtracted
    ResidentResult* res;
};

int sparse_delay_width(int64_t m, int64_t n);
bool sparse_supported(scd_dtype dt, int order, const int64_t* dims, int grid, int* rs, int* cs);
size_t sparse_xbuf_bytes();
hipError_t launch_sparse(const SparseArgs& a, scd_dtype dt, hipStream_t st);
hipError_t launch_transpose(const void* in, void* out, scd_dtype dt, int64_t rows, int64_t cols, hipStream_t st);

// Persistent streaming engine (scd_stream.hip): one launch that streams the remainder once per alternation.
struct PStreamGeometry {
    int grid;        // workgroups (one per compute unit)
    int rpw;         // rows per workgroup
    int cs;          // columns per slice of the hop-1 reduction (multiple of 8, at most 256)
    int lds_rows;    // rows of a workgroup's block kept in LDS for the whole launch
    size_t lds_bytes, xp_bytes, xq_bytes;
};

struct PStreamArgs {
    void* R;                 // m x n (an order-3 tensor n_1 x n_2 x n_3 as m = n_1, n = n_2 n_3)
    int64_t m, n;
    int32_t n2, n3, w2;      // order 3: the two trailing modes and the words of a mode-2 sign vector; else 0
    uint64_t seed;
    int64_t k_start, w_target;
    int32_t max_iters, max_spin;
    int32_t poll_delay;
    uint32_t seq;            // exchange sequence numbers already used
    uint64_t* xp;            // hop 1: [2 parities][grid][n values as tagged words]
    uint64_t* xq;            // hop 2: [2 parities][grid][16 words]
    uint64_t* S;             // term-major outputs; rows k_start.. of S must be zero (bits are OR-ed in)
    uint64_t* T;             // second mode's sign vectors
    uint64_t* S3;            // order 3: third mode's sign vectors (one word per term)
    void* c;
    int32_t* iters;
    double* trace;
    int32_t mw, nw;
    int32_t grid, rpw, cs, lds_rows;
    int32_t profile;         // 1: workgroup 0 times its phases
    int32_t scalars;         // order 3, 1: real last mode ("RGB scalars"): c holds n3 coefficients per term, S3 is not written
    ResidentResult* res;
};

bool pstream_supported(scd_dtype dt, int order, const int64_t* dims, int limit, PStreamGeometry* geo);
hipError_t launch_pstream(const PStreamArgs& a, scd_dtype dt, size_t lds_bytes, hipStream_t st);

// ---- product with a vector from the packed factors (scd_apply.hip) ---------------------------------
struct ApplyPlan {
    int chunks;               // chunks of 4096 input entries
    int parts;                // slices of <t_j, x> per term that the inner pass writes
    int terms_per_wave;       // inner pass
    int splits;               // outer pass: parts the terms are split into
    int64_t terms_per_split;
    int splits_fx;            // outer pass in fixed point (f32): splits of whole tiles of 64 terms
    int64_t terms_per_split_fx;
    size_t off_part, off_ypart, bytes;  // workspace layout
};
void apply_plan(int64_t nin, int64_t nout, int64_t w, ApplyPlan* pl);
hipError_t launch_apply(const uint64_t* in_bits, const uint64_t* out_bits, const void* c, scd_dtype dt, int64_t nin,
                        int64_t nout, int64_t w, const void* x, void* y, void* workspace, hipStream_t st);

// ---- least squares decomposition, Algorithm 6 (scd_lsq.hip) -----------------------------------------
hipError_t launch_lsq_dots(const uint64_t* bits, int64_t k, int64_t nw, int64_t len, const uint64_t* vec, const double* coef,
                           double* out, hipStream_t st);
hipError_t launch_lsq_correct(const uint64_t* bits, int64_t k, int64_t mw, int64_t m, const double* e, const double* base,
                              uint64_t* out_bits, double* abs_parts, double* dot_parts, hipStream_t st);
hipError_t launch_lsq_sum2(const double* a, const double* b, int64_t n, double* out, hipStream_t st);
hipError_t launch_lsq_sumsq(const void* A, scd_dtype dt, int64_t total, double* parts, int nparts, hipStream_t st);
hipError_t launch_lsq_cast(const double* c, int64_t k, scd_dtype dt, void* out, hipStream_t st);
hipError_t launch_lsq_prod(const double* D, int64_t ld, int order, int skip, int64_t k, const double* coef, double* out,
                           hipStream_t st);
hipError_t launch_lsq_kron(const uint64_t* const* signs, const int64_t* dims, int first, int last, int64_t len, uint64_t* out,
                           hipStream_t st);
hipError_t launch_scalars_coef(const double* u, int64_t q, double P, scd_dtype dt, void* c, hipStream_t st);
hipError_t launch_scalars_update(void* r, scd_dtype dt, int64_t total, int64_t q, const uint64_t* lead, const void* c,
                                 double* parts, int nparts, hipStream_t st);
hipError_t launch_lsq_solve(double* L, int64_t ld, int64_t k, const double* g, double diag, const double* bvec, double* yv,
                            double* c, double* work, double fro0sq, double* trace_out, int* status, hipStream_t st);

// ---- launchers implemented in scd_kernels.hip ----------------------------------------------------
hipError_t launch_rowpass(const RowPassArgs& a, scd_dtype dt, int grid, int variant, hipStream_t st);
hipError_t launch_reduce(const ReduceArgs& a, bool f32_partials, hipStream_t st);
hipError_t launch_kron(const KronArgs& a, hipStream_t st);
hipError_t launch_pack(const void* values, scd_dtype dt, int64_t n, uint64_t* bits, hipStream_t st);
hipError_t launch_unpack(const uint64_t* bits, int64_t n, scd_dtype dt, void* values, hipStream_t st);
hipError_t launch_rng(uint64_t seed, uint64_t term, uint32_t mode, int64_t n, uint64_t* bits, hipStream_t st);
hipError_t launch_kron_terms(int order, const int64_t* dims, const uint64_t* const* signs, int64_t w,
                             uint64_t* out, int64_t cols, hipStream_t st);
hipError_t launch_expand(const uint64_t* S, const uint64_t* T, const void* c, scd_dtype dt, int64_t m,
                         int64_t n, int64_t w, void* out, hipStream_t st);
hipError_t launch_halfstep(const void* R, scd_dtype dt, int64_t m, int64_t n, int rows_per_wg, int grid, int do_rows,
                           const uint64_t* sumbits, const uint64_t* rowbits, void* partials, double* u, hipStream_t st);
hipError_t launch_reduce_plain(const void* partials, scd_dtype dt, int nparts, int64_t cols, double* W, uint64_t* bits,
                               double* cparts, hipStream_t st);
hipError_t launch_sum_parts(const double* parts, int n, double* out, hipStream_t st);
hipError_t launch_stream_read(const void* x, int64_t bytes, int grid, float* sink, hipStream_t st);
hipError_t launch_stream_copy(const void* x, void* y, int64_t bytes, int grid, hipStream_t st);
hipError_t launch_exchange_probe(int which, int grid, uint64_t* buf, unsigned* counter, int rounds, int group,
                                 int max_spin, unsigned* err, float* out, hipStream_t st);
bool fast_rowpass_supported(scd_dtype dt, int64_t cols, int level);

}  // namespace scd
