/*
 * scd.h -- C ABI of the MI355X signed cut decomposition library (libscd.so).
 *
 * Method: "Efficient 1-bit tensor approximations", arXiv 2410.01799.
 * A width-w signed cut decomposition of a matrix A (m x n) is
 *        A - R_w = sum_{j<w} c_j * s_j t_j^T ,   s_j in {-1,1}^m, t_j in {-1,1}^n      (abstract, Section 2.2)
 * and of an order-k tensor a (n_1 x ... x n_k)
 *        a - r_w = sum_{j<w} c_j * s_j^(1) (x) ... (x) s_j^(k)                          (Section 5.2).
 * The library builds it with the greedy width loop: Algorithm 4 (Algorithm 12 for tensors)
 * finds one term by alternating s = sgn(R t), t = sgn(R^T s) until <s, R t> stops increasing,
 * Algorithm 5 (Algorithm 13) subtracts it from the remainder and repeats.
 *
 * Conventions shared by every entry point
 *  - Every data pointer is a DEVICE pointer (HIP global memory on the current device) unless the
 *    argument is documented "host".  The caller owns every buffer it passes; the library neither
 *    frees nor keeps them after the call returns.  The library owns only scd_ctx internals.
 *  - Arrays are dense row-major, last mode fastest.  A matrix is order 2, dims = {m, n}.
 *  - dtype: SCD_F32 (float) or SCD_F64 (double) for the input, the remainder and the coefficients.
 *  - Sign vectors are bitsets of uint64 words (Section 3.1: a 1 bit stands for -1).  Element
 *    64p+q is bit q (least significant first) of word p; a vector of length n takes
 *    ceil(n/64) words; padding bits are 0.  Sign matrices are term-major: term j of mode i
 *    starts at word j*ceil(dims[i]/64).
 *  - sgn(x) = -1 iff x < 0 (both zeros give +1).
 *  - Coefficients are normalised, c_j = <s_j, R_{j-1} t_j> / (product of dims), which is what the
 *    definition above needs; Algorithm 5 line 10 divides by mn at the update, the same sequence.
 *  - The random start t_0 of Algorithm 4 line 2 (Algorithm 12 line 1) for (seed, term, mode) is
 *    word p = mix(mix(mix(seed ^ G*(term+1)) + H*(mode+1)) + K*(p+1)) with mix the SplitMix64
 *    finaliser and G,H,K = 0x9E3779B97F4A7C15, 0xD1B54A32D192ED03, 0x8CB92BA72F3D8DD7; modes are
 *    0-based, the matrix t_0 is mode 1; padding bits cleared.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls are
 *    synchronous: results are complete in the caller's buffers when the call returns.
 *  - Return value: SCD_OK (0) or a negative scd_status; SCD_WMAXITER (positive) is a warning:
 *    results are valid but some term ended on the iteration cap instead of on the test of
 *    Algorithm 4 line 8.  No call aborts or throws.  Calls on one context must not overlap.
 */
#ifndef SCD_H
#define SCD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SCD_F32 = 0, SCD_F64 = 1 } scd_dtype;

typedef enum {
    SCD_OK = 0,
    SCD_WMAXITER = 1,    /* warning: a term stopped on the iteration cap */
    SCD_EINVAL = -1,     /* null pointer, order < 2 or > SCD_MAX_ORDER, dim < 1, w < 0, bad dtype */
    SCD_ENOMEM = -2,     /* device or host allocation failed */
    SCD_EHIP = -3,       /* a HIP call failed; scd_last_hip_error() gives its code */
    SCD_EFULL = -4,      /* the context already holds w_capacity terms */
    SCD_ENONFINITE = -5, /* the input (or a remainder given to the context) holds NaN or Inf */
    SCD_ENODEVICE = -6,  /* no usable HIP device */
    SCD_ETIMEOUT = -7,   /* a bounded device-side wait ran out (workgroups of a persistent launch were not all
                            resident); the context refuses further steps until scd_set_remainder */
    SCD_ESINGULAR = -8,  /* scd_lsq_decompose: a new term lies in the span of the earlier ones (normal equations
                            singular to working precision) */
    SCD_ETOOBIG = -9     /* scd_col_signed_sum_noalloc: the input needs more than SCD_NOALLOC_SCRATCH_BYTES */
} scd_status;

#define SCD_MAX_ORDER 8
#define SCD_DEFAULT_MAX_ITERS 4096
#define SCD_LSQ_MAX_WIDTH 4096
#define SCD_NOALLOC_SCRATCH_BYTES (24u << 20) /* fixed work space of scd_col_signed_sum_noalloc, per device */

typedef struct scd_ctx scd_ctx; /* opaque: remainder, scratch, outputs so far, position in the random stream */

/* ---- one-shot decomposition (Algorithm 5 / Algorithm 13) --------------------------------------
 * A        in : order-`order` array of `dt`, dims[order] (host array); not modified.
 * w        in : number of terms (>= 0).          seed: key of the random starts.
 * signs    in : host array of `order` device pointers; signs[i] receives w*ceil(dims[i]/64) words
 *               (matrix: signs[0] = S_w, signs[1] = T_w).
 * c        out: w coefficients of `dt`.
 * fro_trace out: w+1 doubles, ||R_0||_F .. ||R_w||_F, each computed from the remainder itself.
 * iters    out: optional (NULL ok), w int32: alternations (sweeps) each term took. */
int scd_decompose(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, uint64_t seed,
                  void* stream, uint64_t* const* signs, void* c, double* fro_trace, int32_t* iters);

/* ---- stateful form ---------------------------------------------------------------------------
 * scd_create copies A into an internal remainder R_0, computes ||R_0||_F and is ready for term 0.
 * w_capacity bounds the number of terms the context can hold. */
int scd_create(scd_ctx** out, const void* A, scd_dtype dt, int order, const int64_t* dims,
               int64_t w_capacity, uint64_t seed, void* stream);
void scd_destroy(scd_ctx* ctx);

/* Iteration cap of Algorithm 4's loop (the paper's loop is unbounded); default SCD_DEFAULT_MAX_ITERS. */
int scd_set_max_iters(scd_ctx* ctx, int32_t max_iters);

/* Share of the device for this context: its persistent launches take at most `workgroups` workgroups
 * (one per compute unit; 16 or more; 0 = the whole device, the default).
 * The matrices of a model are decomposed independently of one another (Section 4.2), and one greedy
 * decomposition is bound by the latency of its alternations, not by bandwidth: contexts with a share,
 * driven from different host threads on different streams, run side by side and fill each other's
 * waits.  The library serialises persistent launches of one process that would not fit together.
 * The results of a context do not depend on what runs beside it; they may differ in near-tie signs
 * from those of another share (the summation order follows the number of workgroups).
 * Call it between runs, never while another thread uses the context.  May allocate (SCD_ENOMEM). */
int scd_set_workgroups(scd_ctx* ctx, int workgroups);

/* Per-context options.  Everything that selects an engine or tunes one is set here, per context, between
 * runs; the library reads no environment variable.  scd_set_option returns SCD_EINVAL for an unknown option or
 * a value outside its range, and may allocate when it switches an engine on (SCD_ENOMEM). */
typedef enum {
    SCD_OPT_RESIDENT = 0,           /* 0/1 (default 1): the register-resident engine may serve this context */
    SCD_OPT_SPARSE = 1,             /* 0/1 (default 1): the sparse engine (Section 3.1) may serve this context */
    SCD_OPT_SPARSE_MIN_MIB = 2,     /* smallest remainder, in MiB, that the sparse engine takes on a whole device
                                       (default 48; 0 = any size) */
    SCD_OPT_SPARSE_DELAY_WIDTH = 3, /* length of the list of pending terms (Section 3.2): 4..32 (default 8, the
                                       measured optimum; the paper's CPU value is 32), 0 = subtract at once */
    SCD_OPT_ROWPASS_KERNEL = 4,     /* launch-stream engine: 1 = register-tiled row pass where the shape allows
                                       (default), 0 = the generic kernel */
    SCD_OPT_POLL_DELAY = 5,         /* persistent engines: sleep units between publishing and the first read of
                                       the partners' data (default 16) */
    SCD_OPT_MAX_SPIN = 6,           /* persistent engines: re-reads of stale exchange data after which a wait gives
                                       up (default 2^22; 0 = give up at the first stale read: for tests of the
                                       SCD_ETIMEOUT path, every workgroup still exits normally) */
    SCD_OPT_SWEEP_BATCH = 7,        /* launch-stream engine: sweeps enqueued between two looks at the device
                                       state (default 64) */
    SCD_OPT_VERBOSE = 8,            /* 0/1: persistent engines print counters of each launch to stderr */
    SCD_OPT_PERSISTENT_STREAM = 9,  /* 0/1 (default 1): matrices that neither persistent engine above takes are
                                       streamed by one persistent launch instead of a launch per alternation */
    SCD_OPT_COUNT = 10
} scd_option;
int scd_set_option(scd_ctx* ctx, int option, int64_t value);
int scd_get_option(const scd_ctx* ctx, int option, int64_t* value /* host */);

/* Advance exactly one term (Algorithm 5 lines 6-10): greedy cut from the keyed random start of the
 * current term, append (s, t, c), update the remainder, record ||R||_F. */
int scd_step(scd_ctx* ctx);
/* Advance n terms (n >= 0) without returning to the host in between. */
int scd_run(scd_ctx* ctx, int64_t n);
/* Test hook: one term whose start is given by the caller instead of the random stream.
 * init_signs: host array of `order` device pointers to bitsets; entry 0 is ignored (Algorithm 4
 * overwrites s_0 before reading it) and may be NULL. */
int scd_step_from(scd_ctx* ctx, const uint64_t* const* init_signs);

int scd_width(const scd_ctx* ctx, int64_t* k /* host */);
/* Copy out the first k = scd_width() terms; layouts as in scd_decompose (fro_trace gets k+1 values).
 * Any of signs / c / fro_trace / iters may be NULL to skip it. */
int scd_results(const scd_ctx* ctx, uint64_t* const* signs, void* c, double* fro_trace, int32_t* iters);
/* Copy the current remainder R_k out (same dtype and shape as A), or replace it.  Replacing keeps
 * k and the results so far, recomputes ||R_k||_F and restarts the current term. */
int scd_remainder(const scd_ctx* ctx, void* R_out);
int scd_set_remainder(scd_ctx* ctx, const void* R_in);

/* ---- half steps of Algorithm 4 on caller data (lines 5 and 6-7) --------------------------------
 * Row signed sum: u = R t (m doubles, optional) and s = sgn(u) packed (ceil(m/64) words, optional).
 * Column signed sum: v = R^T s (n doubles, optional), t = sgn(v) packed (optional) and
 * c = sum_l |v_l| = <s, R t> (one double, optional; not normalised).  R is m x n of `dt`. */
int scd_row_signed_sum(const void* R, scd_dtype dt, int64_t m, int64_t n, const uint64_t* tbits,
                       void* stream, double* u, uint64_t* sbits);
int scd_col_signed_sum(const void* R, scd_dtype dt, int64_t m, int64_t n, const uint64_t* sbits,
                       void* stream, double* v, uint64_t* tbits, double* c);

/* The column half step for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same geometry and therefore the
 * same bits in v, tbits and c as scd_col_signed_sum, but
 *  - the per-workgroup partial column sums and the partial sums of |v| live in a fixed work space of
 *    SCD_NOALLOC_SCRATCH_BYTES that is part of the library's code object (one copy per device, held until the
 *    process ends); the call allocates and frees nothing;
 *  - the call only enqueues its three launches on `stream` and returns: v, tbits and c are complete once the
 *    stream has reached that point (the caller synchronises, or orders later work on the same stream);
 *  - inputs with 256 + 256*ceil(ceil(n/64)/32) + ceil(m / ceil(m/1024)) * n * sizeof(dt) bytes of work space above
 *    the limit are refused with SCD_ETOOBIG before anything is enqueued (4096 x 4096 f32 fits; f64 does not);
 *  - every call on a device shares that device's work space, which keeps the previous call's contents (each call
 *    overwrites all it reads, nothing needs clearing): calls that overlap in time on one device race, also from
 *    different streams or threads.  Order them on one stream or with events.
 * The device is the current one at the time of the call; R, sbits and the outputs must live on it. */
int scd_col_signed_sum_noalloc(const void* R, scd_dtype dt, int64_t m, int64_t n, const uint64_t* sbits,
                               void* stream, double* v, uint64_t* tbits, double* c);

/* ---- expansion (the definition, Section 2.2 / 5.2) ---------------------------------------------
 * out (dtype dt, dims) = sum_{j<w} c_j * tensor product of term j's sign vectors.  Per entry the
 * terms are added in the order j = 0..w-1 into one f64 accumulator, rounded once to dt, so the
 * result is reproducible bit for bit.  signs: host array of `order` device pointers. */
int scd_expand(const uint64_t* const* signs, const void* c, scd_dtype dt, int order, const int64_t* dims,
               int64_t w, void* stream, void* out);

/* ---- least squares decomposition (Algorithm 6, Section 3.3) --------------------------------------
 * For k = 0..w-1: greedy signed cut (Algorithm 4) of R_k = A - S_k diag(c_k) T_k^T from the keyed random start
 * of term k, append its (s, t), then refit ALL coefficients: c_{k+1} = argmin ||A - S_{k+1} diag(c) T_{k+1}^T||_F
 * by the normal equations of Section 3.3 (Gram matrix from popcounts of the bitsets, Cholesky factor grown by a
 * row per term, f64).  The remainder is kept implicit, A is not modified.  Matrices only.
 * A: device, m x n row-major of dt.  S, T: device out, term-major bitsets as in scd_decompose.  c: device out,
 * w values of dt: the FINAL coefficients c_w of all terms (they are direct coefficients of s_j t_j^T, like the
 * normalised c of scd_decompose).  fro_trace: device out, w + 1 doubles, ||A - S_k diag(c_k) T_k^T||_F for
 * k = 0..w.  iters: device out, optional.  w <= SCD_LSQ_MAX_WIDTH (the factor takes 8 w^2 bytes).
 * Allocates its work space on the device and frees it before returning; synchronous on stream.
 * Returns SCD_OK, SCD_WMAXITER, or SCD_EINVAL / SCD_ENOMEM / SCD_EHIP / SCD_ENONFINITE / SCD_ESINGULAR. */
int scd_lsq_decompose(const void* A, scd_dtype dt, int64_t m, int64_t n, int64_t w, uint64_t seed, int32_t max_iters,
                      void* stream, uint64_t* S, uint64_t* T, void* c, double* fro_trace, int32_t* iters);

/* The same for a tensor of order 2..SCD_MAX_ORDER (Algorithm 14, Section 5.3): axial greedy cut (Algorithm 12) of
 * a - S_k c_k from the keyed random start of term k, then all coefficients refitted.  dims: host array; A: device,
 * row-major, last mode fastest; signs: host array of `order` device pointers, term-major bitsets as in
 * scd_decompose; the other arguments and the status codes as above.  Every mode step makes its own pass over the
 * tensor (the remainder is implicit, so no contracted copy can be reused): meant for small and medium tensors. */
int scd_lsq_decompose_tensor(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, uint64_t seed,
                             int32_t max_iters, void* stream, uint64_t* const* signs, void* c, double* fro_trace,
                             int32_t* iters);

/* ---- real last mode ("RGB scalars", Section 5) ----------------------------------------------------
 * a - r_w = sum_j (s_j^(1) x ... x s_j^(k-1)) x c_j with sign vectors for every mode but the last and a real
 * vector c_j over the last mode (the three colour channels of the paper's image).  The paper names the variant
 * without an algorithm; this entry point takes each term from the axial greedy cut of Algorithm 12 on the
 * whole remainder (keyed random start as in Algorithm 13) and then replaces the last mode's sign vector and
 * the scalar by the real vector that is optimal for the other modes' sign vectors:
 *     c_j[ch] = < s^(1) x ... x s^(k-1), r_j[..., ch] > / (n_1 ... n_{k-1}),   r_{j+1} = r_j - (s^(1) x ...) x c_j.
 * A: device, order >= 2, row-major, last mode fastest, not modified.  signs: host array of order - 1 device
 * pointers (modes 1..k-1), term-major bitsets as in scd_decompose.  c: device out, w * dims[order-1] values of
 * dt, term-major.  fro_trace: device out, w + 1 doubles.  iters: device out, optional (sweeps per term).
 * The remainder is kept in dt; allocates its work space and frees it before returning; synchronous on stream.
 * Returns SCD_OK, SCD_WMAXITER, or SCD_EINVAL / SCD_ENOMEM / SCD_EHIP / SCD_ENONFINITE. */
int scd_decompose_scalars(const void* A, scd_dtype dt, int order, const int64_t* dims, int64_t w, uint64_t seed,
                          int32_t max_iters, void* stream, uint64_t* const* signs, void* c, double* fro_trace,
                          int32_t* iters);

/* Product of a matrix decomposition with a vector, straight from the packed factors, without expanding
 * the matrix (Section 6.1, Question A):
 *   transpose == 0:  y = (sum_{j<w} c_j s_j t_j^T) x      x: n entries, y: m entries
 *   transpose != 0:  y = (sum_{j<w} c_j s_j t_j^T)^T x    x: m entries, y: n entries
 * computed as z_j = c_j <t_j, x> and y = sum_j z_j s_j, every sum in a fixed order, y rounded once to dt.
 * dt = SCD_F64: all sums in f64.  dt = SCD_F32: both sums are formed in block fixed point (each chunk of 4096
 * entries of x, and the z_j of each split of at most 2048 terms, scaled by a power of two and rounded to
 * integers below 2^30: at most max|x| 2^-30 per entry and max|z| 2^-30 per term, exact integer sums
 * afterwards), the rest in f64.  Non-finite entries of x give NaN.  S, T: device, term-major bitsets as scd_decompose writes them (w * ceil(m/64) and
 * w * ceil(n/64) words, padding bits 0); c, x, y: device, dtype dt; x and y must not overlap.
 * nvec >= 1 vectors are taken one after the other: x is nvec rows of the input length, y nvec rows of the
 * output length.  workspace: device, at least scd_apply_workspace_bytes(m, n, w) bytes, 8-byte aligned,
 * owned by the caller and free again on return; the call allocates nothing and is synchronous on stream.
 * w == 0 gives y = 0.  SCD_EINVAL on null pointers, negative sizes, m or n above 2^31, a workspace that
 * is too small. */
size_t scd_apply_workspace_bytes(int64_t m, int64_t n, int64_t w);
int scd_apply(const uint64_t* S, const uint64_t* T, const void* c, scd_dtype dt, int64_t m, int64_t n, int64_t w,
              int transpose, const void* x, int64_t nvec, void* y, void* workspace, size_t workspace_bytes,
              void* stream);

/* ---- bitsets (Section 3.1) -------------------------------------------------------------------- */
int scd_pack(const void* values, scd_dtype dt, int64_t n, void* stream, uint64_t* bits);   /* x < 0 -> 1 */
int scd_unpack(const uint64_t* bits, int64_t n, scd_dtype dt, void* stream, void* values); /* 1 -> -1.0 */
/* The keyed random start of Algorithm 4 line 2 for (seed, term, mode), n signs, padding cleared. */
int scd_rng_signs(uint64_t seed, uint64_t term, uint32_t mode, int64_t n, void* stream, uint64_t* bits);

/* ---- diagnostics ------------------------------------------------------------------------------ */
const char* scd_strerror(int code);
int scd_last_hip_error(void);        /* hipError_t of the most recent SCD_EHIP on this thread */
#ifdef __cplusplus
}
#endif
#endif /* SCD_H */
