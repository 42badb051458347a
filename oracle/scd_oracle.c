/*
 * scd_oracle.c -- plain f64 CPU oracle for the greedy signed cut decomposition.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * method computes.  It is used by the tests, by the smoke check and by the benchmark's CPU
 * baseline leg; the GPU library never links, loads or calls it, and it shares no code with it.
 *
 * Paper: "Efficient 1-bit tensor approximations" (Riasanovsky, El Kazdadi), arXiv 2410.01799.
 *   - Section 3.1, Algorithm 4  GREEDY SIGNED CUT          -> scdo_greedy_signed_cut
 *   - Section 3.2, Algorithm 5  GREEDY DECOMPOSITION       -> scdo_decompose
 *   - Section 3.2, Frobenius identity                      -> checked by the tests, not used here
 *   - Section 3.3, Algorithm 6  LEAST SQUARES DECOMPOSITION-> scdo_lsq_coefficients, scdo_lsq_decompose
 *   - Section 5.1, Algorithm 12 AXIAL GREEDY CUT           -> scdo_axial_greedy_cut
 *   - Section 5.2, Algorithm 13 TENSOR GREEDY DECOMPOSITION-> scdo_tensor_decompose
 *   - Section 5.3, Algorithm 14 TENSOR LEAST SQUARES       -> scdo_tensor_lsq_coefficients,
 *                                                             scdo_tensor_lsq_decompose
 *   - Section 5, "RGB scalars": sum_j s_j (x) t_j (x) c_j with real c_j -> scdo_scalars_decompose
 *   - Section 2.2 / 5.2 definition  a - r_w = sum_j c_j s_j -> scdo_expand
 *   - Section 6.1 (Question A) product of the decomposition with a vector, without expanding it
 *                                                          -> scdo_apply
 *   - Section 2.2 signed cut norm (max over sign vectors)  -> scdo_bruteforce_signed_cut_norm
 *   - Section 3.1 sign bitsets (a 1 bit stands for -1)     -> scdo_pack / scdo_unpack
 *
 * Everything is double precision.  Products with +-1 are written as multiplications: this is
 * the definition, not an optimisation.  No blocking, no fusion, no caching of differences.
 *
 * Readings taken where the paper is silent (each also listed in the design document):
 *   - sgn(x) = -1 iff x < 0; both zeros give +1.
 *   - The stored coefficient is the normalised one, c_j = <s,R t>/(mn), so that
 *     A - R_w = sum_j c_j s_j t_j^T holds as the abstract states; Algorithm 5 divides by mn
 *     only at the update, which is the same remainder sequence.
 *   - Algorithm 4 samples s_0 but overwrites it before any use; only t_0 is drawn.
 *   - "sample uniformly" is realised by a stateless counter-based generator keyed by
 *     (seed, term, mode, word), see scdo_rng_word.
 *   - Bitsets are uint64 words, element 64p+q is bit q (LSB first) of word p, padding bits 0.
 *   - An iteration cap (max_iters) guards the unbounded loop of Algorithm 4 / 12.
 *   - "RGB scalars" is named in Section 5 without an algorithm.  Reading: every term is found by the
 *     axial greedy cut of Algorithm 12 on the whole tensor (all modes signs, as for "RGB signs"); the
 *     last mode's sign vector and the scalar are then replaced by the real vector that is optimal for
 *     the other modes' sign vectors, one least-squares coefficient per slice of the last mode.
 *
 * OpenMP pragmas only split loops whose iterations are independent (rows of R t, column
 * ranges of R^T s, rows of the update); the order of every floating point sum is the same
 * for any thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define SCDO_MAX_ORDER 8

/* ---------------------------------------------------------------- threads */

void scdo_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

int scdo_get_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- random signs */

/* 64-bit finaliser of the SplitMix64 generator (Steele, Lea, Flood 2014; public domain
 * constants as published by Vigna). */
static uint64_t mix64(uint64_t z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ull;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBull;
    z ^= z >> 31;
    return z;
}

/* Word `word` of the uniform random sign vector that Algorithm 4 line 2 (Algorithm 12 line 1)
 * draws for term `term`, tensor mode `mode` (0-based; the matrix t_0 is mode 1). */
uint64_t scdo_rng_word(uint64_t seed, uint64_t term, uint32_t mode, uint64_t word)
{
    uint64_t h = mix64(seed ^ (0x9E3779B97F4A7C15ull * (term + 1)));
    h = mix64(h + 0xD1B54A32D192ED03ull * ((uint64_t)mode + 1));
    h = mix64(h + 0x8CB92BA72F3D8DD7ull * (word + 1));
    return h;
}

static int64_t words_for(int64_t n) { return (n + 63) / 64; }

void scdo_rng_signs(uint64_t seed, uint64_t term, uint32_t mode, int64_t n, uint64_t* bits)
{
    int64_t nw = words_for(n);
    for (int64_t p = 0; p < nw; ++p) bits[p] = scdo_rng_word(seed, term, mode, (uint64_t)p);
    if (n % 64) bits[nw - 1] &= (~0ull) >> (64 - n % 64);
}

/* ---------------------------------------------------------------- bitsets (Section 3.1) */

static double sign_at(const uint64_t* bits, int64_t i)
{
    return ((bits[i >> 6] >> (i & 63)) & 1ull) ? -1.0 : 1.0;
}

/* bit = 1  <=>  x < 0  (so +0.0 and -0.0 both give bit 0) */
void scdo_pack(const double* x, int64_t n, uint64_t* bits)
{
    int64_t nw = words_for(n);
    for (int64_t p = 0; p < nw; ++p) bits[p] = 0;
    for (int64_t i = 0; i < n; ++i)
        if (x[i] < 0.0) bits[i >> 6] |= 1ull << (i & 63);
}

void scdo_unpack(const uint64_t* bits, int64_t n, double* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = sign_at(bits, i);
}

/* ---------------------------------------------------------------- matrix products with sign vectors */

/* u = R t,  R is m x n row-major, t given as bits (Algorithm 4 line 5 before the sgn). */
void scdo_row_signed_sum(const double* R, int64_t m, int64_t n, const uint64_t* tbits, double* u)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double acc = 0.0;
        for (int64_t l = 0; l < n; ++l) acc += R[i * n + l] * sign_at(tbits, l);
        u[i] = acc;
    }
}

/* v = R^T s (Algorithm 4 line 6 before the sgn).  Each v_l is summed over i = 0..m-1 in order. */
void scdo_col_signed_sum(const double* R, int64_t m, int64_t n, const uint64_t* sbits, double* v)
{
    for (int64_t l = 0; l < n; ++l) v[l] = 0.0;
#pragma omp parallel
    {
        int64_t lo = 0, hi = n;
#ifdef _OPENMP
        int nt = omp_get_num_threads(), id = omp_get_thread_num();
        lo = n * id / nt;
        hi = n * (id + 1) / nt;
#endif
        for (int64_t i = 0; i < m; ++i) {
            double si = sign_at(sbits, i);
            for (int64_t l = lo; l < hi; ++l) v[l] += R[i * n + l] * si;
        }
    }
}

static double max_abs(const double* x, int64_t n)
{
    double mx = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double a = fabs(x[i]);
        if (a > mx) mx = a;
    }
    return mx;
}

static double min_abs(const double* x, int64_t n)
{
    double mn = INFINITY;
    for (int64_t i = 0; i < n; ++i) {
        double a = fabs(x[i]);
        if (a < mn) mn = a;
    }
    return mn;
}

/* squared Frobenius norm: each row summed in order, then the row sums in order */
double scdo_fro2(const double* R, int64_t rows, int64_t cols)
{
    double* rs = (double*)malloc(sizeof(double) * (size_t)(rows > 0 ? rows : 1));
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < rows; ++i) {
        double acc = 0.0;
        for (int64_t l = 0; l < cols; ++l) acc += R[i * cols + l] * R[i * cols + l];
        rs[i] = acc;
    }
    double tot = 0.0;
    for (int64_t i = 0; i < rows; ++i) tot += rs[i];
    free(rs);
    return tot;
}

/* R <- R - ck * s t^T   (Algorithm 5 line 10 with ck = c/(mn)) */
void scdo_rank1_update(double* R, int64_t m, int64_t n, double ck, const uint64_t* sbits,
                       const uint64_t* tbits)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < m; ++i) {
        double si = sign_at(sbits, i);
        for (int64_t l = 0; l < n; ++l) R[i * n + l] -= ck * si * sign_at(tbits, l);
    }
}

/* ---------------------------------------------------------------- Algorithm 4 */

/*
 * GREEDY SIGNED CUT on R (m x n).
 *   tbits   in: t_0;  out: t_j of the returned triple          (ceil(n/64) words)
 *   sbits   out: s_j                                           (ceil(m/64) words)
 *   c_out   out: c_j = <s_j, R t_j>   (NOT divided by mn)
 *   iters   out: j, the number of alternations performed
 *   c_hist  optional, max_iters doubles: c_1 .. c_j
 *   margin  optional, 2 doubles: min over alternations of min_i |(R t)_i| / max_i |(R t)_i|
 *           and the same for R^T s -- how close any sign decision came to a tie
 * Returns 0, or 1 if the cap max_iters ended the loop.
 */
int scdo_greedy_signed_cut(const double* R, int64_t m, int64_t n, uint64_t* tbits, uint64_t* sbits,
                           double* c_out, int32_t max_iters, int32_t* iters, double* c_hist,
                           double* margin)
{
    double* u = (double*)malloc(sizeof(double) * (size_t)m);
    double* v = (double*)malloc(sizeof(double) * (size_t)n);
    double c_prev = -INFINITY, c = 0.0;
    double mg_u = INFINITY, mg_v = INFINITY;
    int hit_cap = 1;
    int32_t j = 0;

    scdo_row_signed_sum(R, m, n, tbits, u); /* R t_0 */
    while (j < max_iters) {
        ++j;
        {
            double mx = max_abs(u, m);
            if (mx > 0.0 && min_abs(u, m) / mx < mg_u) mg_u = min_abs(u, m) / mx;
            if (mx == 0.0) mg_u = 0.0;
        }
        scdo_pack(u, m, sbits);                 /* line 5: s_j = sgn(R t_{j-1}) */
        scdo_col_signed_sum(R, m, n, sbits, v); /*         R^T s_j              */
        {
            double mx = max_abs(v, n);
            if (mx > 0.0 && min_abs(v, n) / mx < mg_v) mg_v = min_abs(v, n) / mx;
            if (mx == 0.0) mg_v = 0.0;
        }
        scdo_pack(v, n, tbits);                 /* line 6: t_j = sgn(R^T s_j)   */
        scdo_row_signed_sum(R, m, n, tbits, u); /*         R t_j                */
        c = 0.0;                                /* line 7: c_j = <s_j, R t_j>   */
        for (int64_t i = 0; i < m; ++i) c += sign_at(sbits, i) * u[i];
        if (c_hist) c_hist[j - 1] = c;
        if (c <= c_prev) { /* line 8 */
            hit_cap = 0;
            break;
        }
        c_prev = c;
    }
    *c_out = c;
    if (iters) *iters = j;
    if (margin) {
        margin[0] = mg_u;
        margin[1] = mg_v;
    }
    free(u);
    free(v);
    return hit_cap;
}

/* ---------------------------------------------------------------- Algorithm 5 */

/*
 * GREEDY DECOMPOSITION of A (m x n) to width w.
 *   S      out: w * ceil(m/64) words, term-major     T: w * ceil(n/64) words
 *   c      out: w normalised coefficients, A - R_w = sum_j c[j] s_j t_j^T
 *   trace  out: w+1 values ||R_0||_F .. ||R_w||_F
 *   iters  optional out: w alternation counts
 *   margins optional out: 2*w tie margins (see scdo_greedy_signed_cut)
 *   R_out  optional out: the final remainder R_w (m*n)
 * Returns the number of terms that hit the iteration cap.
 */
int scdo_decompose(const double* A, int64_t m, int64_t n, int64_t w, uint64_t seed,
                   int32_t max_iters, uint64_t* S, uint64_t* T, double* c, double* trace,
                   int32_t* iters, double* margins, double* R_out)
{
    int64_t mw = words_for(m), nw = words_for(n);
    size_t bytes = sizeof(double) * (size_t)m * (size_t)n;
    double* R = (double*)malloc(bytes);
    int capped = 0;
    memcpy(R, A, bytes); /* line 1: R_0 = A */
    trace[0] = sqrt(scdo_fro2(R, m, n));
    for (int64_t k = 0; k < w; ++k) {
        uint64_t* sk = S + k * mw;
        uint64_t* tk = T + k * nw;
        double cu;
        int32_t it;
        scdo_rng_signs(seed, (uint64_t)k, 1, n, tk); /* Algorithm 4 line 2 */
        capped += scdo_greedy_signed_cut(R, m, n, tk, sk, &cu, max_iters, &it, NULL,
                                         margins ? margins + 2 * k : NULL);
        c[k] = cu / ((double)m * (double)n);
        if (iters) iters[k] = it;
        scdo_rank1_update(R, m, n, c[k], sk, tk); /* line 10 */
        trace[k + 1] = sqrt(scdo_fro2(R, m, n));
    }
    if (R_out) memcpy(R_out, R, bytes);
    free(R);
    return capped;
}

/* ---------------------------------------------------------------- Algorithm 6 (Section 3.3) */

/*
 * c = argmin || A - sum_{j<k} c_j s_j t_j^T ||_F  (Algorithm 6 line 9) by the normal equations of
 * Section 3.3:  G c = b,  G_ij = <s_i t_i^T, s_j t_j^T>_F,  b_i = <s_i t_i^T, A>_F.  Every inner
 * product is the sum over all entries, written out.  G is solved by Gaussian elimination with partial
 * pivoting.  Returns 0, or 1 if G is singular to working precision (repeated terms).
 */
int scdo_lsq_coefficients(const double* A, int64_t m, int64_t n, int64_t k, const uint64_t* S,
                          const uint64_t* T, double* c)
{
    int64_t mw = words_for(m), nw = words_for(n);
    double* G;
    double* b;
    int singular = 0;
    if (k == 0) return 0;
    G = (double*)malloc(sizeof(double) * (size_t)k * (size_t)k);
    b = (double*)malloc(sizeof(double) * (size_t)k);
    for (int64_t a = 0; a < k; ++a) {
        double acc = 0.0;
        for (int64_t i = 0; i < m; ++i)
            for (int64_t l = 0; l < n; ++l)
                acc += sign_at(S + a * mw, i) * sign_at(T + a * nw, l) * A[i * n + l];
        b[a] = acc;
        for (int64_t q = 0; q <= a; ++q) {
            double g = 0.0;
            for (int64_t i = 0; i < m; ++i) {
                double si = sign_at(S + a * mw, i) * sign_at(S + q * mw, i);
                for (int64_t l = 0; l < n; ++l) g += si * sign_at(T + a * nw, l) * sign_at(T + q * nw, l);
            }
            G[a * k + q] = g;
            G[q * k + a] = g;
        }
    }
    for (int64_t col = 0; col < k; ++col) {
        int64_t piv = col;
        for (int64_t r = col + 1; r < k; ++r)
            if (fabs(G[r * k + col]) > fabs(G[piv * k + col])) piv = r;
        if (fabs(G[piv * k + col]) < 1e-9 * (double)m * (double)n) {
            singular = 1;
            break;
        }
        if (piv != col) {
            for (int64_t q = 0; q < k; ++q) {
                double tmp = G[col * k + q];
                G[col * k + q] = G[piv * k + q];
                G[piv * k + q] = tmp;
            }
            double tb = b[col];
            b[col] = b[piv];
            b[piv] = tb;
        }
        for (int64_t r = col + 1; r < k; ++r) {
            double f = G[r * k + col] / G[col * k + col];
            for (int64_t q = col; q < k; ++q) G[r * k + q] -= f * G[col * k + q];
            b[r] -= f * b[col];
        }
    }
    if (!singular) {
        for (int64_t r = k - 1; r >= 0; --r) {
            double acc = b[r];
            for (int64_t q = r + 1; q < k; ++q) acc -= G[r * k + q] * c[q];
            c[r] = acc / G[r * k + r];
        }
    }
    free(G);
    free(b);
    return singular;
}

/*
 * LEAST SQUARES DECOMPOSITION.  Term k: R_k = A - S_k diag(c_k) T_k^T (line 5, read with the "A -" that
 * the caption's "orthogonal complement of A" requires), greedy signed cut of R_k from the keyed random
 * start of term k (line 6; its value is discarded), append (lines 7-8), new coefficients for ALL terms
 * (line 9).  c gets the final coefficients c_w; trace[k] = ||A - S_k diag(c_k) T_k^T||_F, k = 0..w.
 * Returns the number of terms whose cut hit max_iters, or -1 if the normal equations became singular.
 */
int scdo_lsq_decompose(const double* A, int64_t m, int64_t n, int64_t w, uint64_t seed, int32_t max_iters,
                       uint64_t* S, uint64_t* T, double* c, double* trace, int32_t* iters, double* margins)
{
    int64_t mw = words_for(m), nw = words_for(n);
    size_t bytes = sizeof(double) * (size_t)m * (size_t)n;
    double* R = (double*)malloc(bytes);
    int capped = 0;
    memcpy(R, A, bytes);
    trace[0] = sqrt(scdo_fro2(R, m, n));
    for (int64_t k = 0; k < w; ++k) {
        uint64_t* sk = S + k * mw;
        uint64_t* tk = T + k * nw;
        double cu;
        int32_t it;
        scdo_rng_signs(seed, (uint64_t)k, 1, n, tk);
        capped += scdo_greedy_signed_cut(R, m, n, tk, sk, &cu, max_iters, &it, NULL,
                                         margins ? margins + 2 * k : NULL);
        if (iters) iters[k] = it;
        if (scdo_lsq_coefficients(A, m, n, k + 1, S, T, c)) {
            free(R);
            return -1;
        }
        memcpy(R, A, bytes);
        for (int64_t j = 0; j <= k; ++j) scdo_rank1_update(R, m, n, c[j], S + j * mw, T + j * nw);
        trace[k + 1] = sqrt(scdo_fro2(R, m, n));
    }
    free(R);
    return capped;
}

/* ---------------------------------------------------------------- tensors (Section 5) */

static int64_t total_size(int order, const int64_t* dims)
{
    int64_t N = 1;
    for (int i = 0; i < order; ++i) N *= dims[i];
    return N;
}

/* advance a row-major multi-index (last mode fastest); returns 0 after the last element */
static int next_index(int order, const int64_t* dims, int64_t* idx)
{
    for (int i = order - 1; i >= 0; --i) {
        if (++idx[i] < dims[i]) return 1;
        idx[i] = 0;
    }
    return 0;
}

/*
 * u = a x_mode (tensor product of the sign vectors of all OTHER modes): Algorithm 12 line 8
 * before the sgn.  u has dims[mode] entries; signs[i] is the bitset of mode i.
 */
void scdo_mode_signed_sum(const double* a, int order, const int64_t* dims,
                          const uint64_t* const* signs, int mode, double* u)
{
    int64_t idx[SCDO_MAX_ORDER] = {0};
    int64_t N = total_size(order, dims);
    for (int64_t x = 0; x < dims[mode]; ++x) u[x] = 0.0;
    if (N == 0) return;
    int64_t pos = 0;
    do {
        double sg = 1.0;
        for (int i = 0; i < order; ++i)
            if (i != mode) sg *= sign_at(signs[i], idx[i]);
        u[idx[mode]] += a[pos] * sg;
        ++pos;
    } while (next_index(order, dims, idx));
}

/* <s, a> with s the tensor product of all mode sign vectors (Algorithm 12 line 10) */
double scdo_tensor_inner(const double* a, int order, const int64_t* dims,
                         const uint64_t* const* signs)
{
    int64_t idx[SCDO_MAX_ORDER] = {0};
    int64_t N = total_size(order, dims);
    double acc = 0.0;
    if (N == 0) return 0.0;
    int64_t pos = 0;
    do {
        double sg = 1.0;
        for (int i = 0; i < order; ++i) sg *= sign_at(signs[i], idx[i]);
        acc += a[pos] * sg;
        ++pos;
    } while (next_index(order, dims, idx));
    return acc;
}

/* r <- r - ck * (tensor product of the sign vectors)   (Algorithm 13 line 8, ck = c/prod n_i) */
void scdo_tensor_update(double* r, int order, const int64_t* dims, double ck,
                        const uint64_t* const* signs)
{
    int64_t idx[SCDO_MAX_ORDER] = {0};
    int64_t N = total_size(order, dims);
    if (N == 0) return;
    int64_t pos = 0;
    do {
        double sg = 1.0;
        for (int i = 0; i < order; ++i) sg *= sign_at(signs[i], idx[i]);
        r[pos] -= ck * sg;
        ++pos;
    } while (next_index(order, dims, idx));
}

/*
 * AXIAL GREEDY CUT.  signs[i] in: s_{0,i} (mode 0's is never read), out: s_{j,i}.
 * c_out = <s_j, a> (not normalised).  margin: optional, `order` doubles, the per-mode tie margin.
 * Returns 0, or 1 if max_iters ended the loop.
 */
int scdo_axial_greedy_cut(const double* a, int order, const int64_t* dims, uint64_t* const* signs,
                          double* c_out, int32_t max_iters, int32_t* iters, double* c_hist,
                          double* margin)
{
    int64_t maxd = 0;
    for (int i = 0; i < order; ++i)
        if (dims[i] > maxd) maxd = dims[i];
    double* u = (double*)malloc(sizeof(double) * (size_t)(maxd > 0 ? maxd : 1));
    double c_prev = -INFINITY, c = 0.0;
    int hit_cap = 1;
    int32_t j = 0;
    if (margin)
        for (int i = 0; i < order; ++i) margin[i] = INFINITY;
    while (j < max_iters) {
        ++j;
        for (int i = 0; i < order; ++i) { /* lines 4-8: modes < i already new, modes > i old */
            scdo_mode_signed_sum(a, order, dims, (const uint64_t* const*)signs, i, u);
            if (margin) {
                double mx = max_abs(u, dims[i]);
                double mg = mx > 0.0 ? min_abs(u, dims[i]) / mx : 0.0;
                if (mg < margin[i]) margin[i] = mg;
            }
            scdo_pack(u, dims[i], signs[i]);
        }
        c = scdo_tensor_inner(a, order, dims, (const uint64_t* const*)signs); /* line 10 */
        if (c_hist) c_hist[j - 1] = c;
        if (c <= c_prev) {
            hit_cap = 0;
            break;
        }
        c_prev = c;
    }
    *c_out = c;
    if (iters) *iters = j;
    free(u);
    return hit_cap;
}

/*
 * TENSOR GREEDY DECOMPOSITION.  signs_out[i]: w * ceil(dims[i]/64) words, term-major.
 * c: w normalised coefficients (a - r_w = sum_j c[j] * tensor product of term j's signs).
 * trace: w+1 Frobenius norms.  margins: optional, order*w.  r_out: optional final remainder.
 */
int scdo_tensor_decompose(const double* a, int order, const int64_t* dims, int64_t w,
                          uint64_t seed, int32_t max_iters, uint64_t* const* signs_out, double* c,
                          double* trace, int32_t* iters, double* margins, double* r_out)
{
    int64_t N = total_size(order, dims);
    size_t bytes = sizeof(double) * (size_t)N;
    double* r = (double*)malloc(bytes ? bytes : 8);
    uint64_t* cur[SCDO_MAX_ORDER];
    int capped = 0;
    memcpy(r, a, bytes);
    trace[0] = sqrt(scdo_fro2(r, 1, N));
    for (int64_t k = 0; k < w; ++k) {
        double cu;
        int32_t it;
        for (int i = 0; i < order; ++i) {
            cur[i] = signs_out[i] + k * words_for(dims[i]);
            scdo_rng_signs(seed, (uint64_t)k, (uint32_t)i, dims[i], cur[i]); /* Alg 12 line 1 */
        }
        capped += scdo_axial_greedy_cut(r, order, dims, cur, &cu, max_iters, &it, NULL,
                                        margins ? margins + order * k : NULL);
        c[k] = cu / (double)N;
        if (iters) iters[k] = it;
        scdo_tensor_update(r, order, dims, c[k], (const uint64_t* const*)cur);
        trace[k + 1] = sqrt(scdo_fro2(r, 1, N));
    }
    if (r_out) memcpy(r_out, r, bytes);
    free(r);
    return capped;
}

/* ---------------------------------------------------------------- Algorithm 14 (Section 5.3) */

/* Gaussian elimination with partial pivoting on the k x k system G c = b (G, b are overwritten).
 * Returns 1 if a pivot falls below tol. */
static int solve_dense(double* G, double* b, int64_t k, double tol, double* c)
{
    for (int64_t col = 0; col < k; ++col) {
        int64_t piv = col;
        for (int64_t r = col + 1; r < k; ++r)
            if (fabs(G[r * k + col]) > fabs(G[piv * k + col])) piv = r;
        if (fabs(G[piv * k + col]) < tol) return 1;
        if (piv != col) {
            for (int64_t q = 0; q < k; ++q) {
                double tmp = G[col * k + q];
                G[col * k + q] = G[piv * k + q];
                G[piv * k + q] = tmp;
            }
            double tb = b[col];
            b[col] = b[piv];
            b[piv] = tb;
        }
        for (int64_t r = col + 1; r < k; ++r) {
            double f = G[r * k + col] / G[col * k + col];
            for (int64_t q = col; q < k; ++q) G[r * k + q] -= f * G[col * k + q];
            b[r] -= f * b[col];
        }
    }
    for (int64_t r = k - 1; r >= 0; --r) {
        double acc = b[r];
        for (int64_t q = r + 1; q < k; ++q) acc -= G[r * k + q] * c[q];
        c[r] = acc / G[r * k + r];
    }
    return 0;
}

/*
 * c = argmin || a - sum_{j<k} c_j (tensor product of term j's sign vectors) ||_2  (Algorithm 14 line 8),
 * by the normal equations as in Section 3.3: G_ij = <S_i, S_j>, b_i = <S_i, a>, every inner product summed
 * over all entries of the tensor.  signs[i]: k * ceil(dims[i]/64) words, term-major.
 */
int scdo_tensor_lsq_coefficients(const double* a, int order, const int64_t* dims, int64_t k,
                                 const uint64_t* const* signs, double* c)
{
    int64_t N = total_size(order, dims);
    int64_t nw[SCDO_MAX_ORDER];
    double* G;
    double* b;
    int singular;
    if (k == 0) return 0;
    for (int i = 0; i < order; ++i) nw[i] = words_for(dims[i]);
    G = (double*)malloc(sizeof(double) * (size_t)k * (size_t)k);
    b = (double*)malloc(sizeof(double) * (size_t)k);
    for (int64_t p = 0; p < k; ++p) {
        const uint64_t* sp[SCDO_MAX_ORDER];
        for (int i = 0; i < order; ++i) sp[i] = signs[i] + p * nw[i];
        b[p] = scdo_tensor_inner(a, order, dims, sp);
        for (int64_t q = 0; q <= p; ++q) {
            int64_t idx[SCDO_MAX_ORDER] = {0};
            double g = 0.0;
            if (N > 0) do {
                double sg = 1.0;
                for (int i = 0; i < order; ++i)
                    sg *= sign_at(sp[i], idx[i]) * sign_at(signs[i] + q * nw[i], idx[i]);
                g += sg;
            } while (next_index(order, dims, idx));
            G[p * k + q] = g;
            G[q * k + p] = g;
        }
    }
    singular = solve_dense(G, b, k, 1e-9 * (double)N, c);
    free(G);
    free(b);
    return singular;
}

/*
 * TENSOR LEAST SQUARES.  Term k: r_k = a - S_k c_k (line 4), axial greedy cut of r_k from the keyed
 * random start of term k (line 5, every mode drawn as in Algorithm 13), append (lines 6-7), new
 * coefficients for all terms (line 8).  Outputs as scdo_tensor_decompose, with c the final coefficients.
 * Returns the number of capped terms, or -1 if the normal equations became singular.
 */
int scdo_tensor_lsq_decompose(const double* a, int order, const int64_t* dims, int64_t w, uint64_t seed,
                              int32_t max_iters, uint64_t* const* signs_out, double* c, double* trace,
                              int32_t* iters, double* margins)
{
    int64_t N = total_size(order, dims);
    size_t bytes = sizeof(double) * (size_t)N;
    double* r = (double*)malloc(bytes ? bytes : 8);
    uint64_t* cur[SCDO_MAX_ORDER];
    int capped = 0;
    memcpy(r, a, bytes);
    trace[0] = sqrt(scdo_fro2(r, 1, N));
    for (int64_t k = 0; k < w; ++k) {
        double cu;
        int32_t it;
        for (int i = 0; i < order; ++i) {
            cur[i] = signs_out[i] + k * words_for(dims[i]);
            scdo_rng_signs(seed, (uint64_t)k, (uint32_t)i, dims[i], cur[i]);
        }
        capped += scdo_axial_greedy_cut(r, order, dims, cur, &cu, max_iters, &it, NULL,
                                        margins ? margins + order * k : NULL);
        if (iters) iters[k] = it;
        if (scdo_tensor_lsq_coefficients(a, order, dims, k + 1, (const uint64_t* const*)signs_out, c)) {
            free(r);
            return -1;
        }
        memcpy(r, a, bytes);
        for (int64_t j = 0; j <= k; ++j) {
            const uint64_t* sj[SCDO_MAX_ORDER];
            for (int i = 0; i < order; ++i) sj[i] = signs_out[i] + j * words_for(dims[i]);
            scdo_tensor_update(r, order, dims, c[j], sj);
        }
        trace[k + 1] = sqrt(scdo_fro2(r, 1, N));
    }
    free(r);
    return capped;
}

/* ---------------------------------------------------------------- real last mode ("RGB scalars", Section 5) */

/*
 * a - r_w = sum_j (s_j^(1) x ... x s_j^(k-1)) x c_j with c_j in R^{n_k}.  Term j: axial greedy cut of
 * r_j (Algorithm 12, keyed random start as in Algorithm 13); P = n_1 ... n_{k-1};
 *   c_j[ch] = < s^(1) x ... x s^(k-1), r_j[..., ch] > / P,      r_{j+1}[..., ch] = r_j[..., ch] - c_j[ch] (s^(1) x ...).
 * signs_out: `order` bitset arrays as in scdo_tensor_decompose (the last mode's is the cut's sign vector,
 * equal to sgn(c_j); it is not part of the decomposition).  cvec: w * n_k coefficients, term-major.
 */
int scdo_scalars_decompose(const double* a, int order, const int64_t* dims, int64_t w, uint64_t seed,
                           int32_t max_iters, uint64_t* const* signs_out, double* cvec, double* trace,
                           int32_t* iters, double* margins)
{
    int64_t N = total_size(order, dims);
    int64_t q = dims[order - 1];
    int64_t P = N / q;
    size_t bytes = sizeof(double) * (size_t)N;
    double* r = (double*)malloc(bytes ? bytes : 8);
    uint64_t* cur[SCDO_MAX_ORDER];
    int capped = 0;
    memcpy(r, a, bytes);
    trace[0] = sqrt(scdo_fro2(r, 1, N));
    for (int64_t k = 0; k < w; ++k) {
        double cu;
        int32_t it;
        for (int i = 0; i < order; ++i) {
            cur[i] = signs_out[i] + k * words_for(dims[i]);
            scdo_rng_signs(seed, (uint64_t)k, (uint32_t)i, dims[i], cur[i]);
        }
        capped += scdo_axial_greedy_cut(r, order, dims, cur, &cu, max_iters, &it, NULL,
                                        margins ? margins + order * k : NULL);
        if (iters) iters[k] = it;
        for (int64_t ch = 0; ch < q; ++ch) {
            int64_t idx[SCDO_MAX_ORDER] = {0};
            double acc = 0.0;
            for (int64_t p = 0; p < P; ++p) { /* p runs over the leading modes, last of them fastest */
                double sg = 1.0;
                for (int i = 0; i + 1 < order; ++i) sg *= sign_at(cur[i], idx[i]);
                acc += sg * r[p * q + ch];
                for (int i = order - 2; i >= 0; --i) {
                    if (++idx[i] < dims[i]) break;
                    idx[i] = 0;
                }
            }
            cvec[k * q + ch] = acc / (double)P;
        }
        {
            int64_t idx[SCDO_MAX_ORDER] = {0};
            for (int64_t p = 0; p < P; ++p) {
                double sg = 1.0;
                for (int i = 0; i + 1 < order; ++i) sg *= sign_at(cur[i], idx[i]);
                for (int64_t ch = 0; ch < q; ++ch) r[p * q + ch] -= cvec[k * q + ch] * sg;
                for (int i = order - 2; i >= 0; --i) {
                    if (++idx[i] < dims[i]) break;
                    idx[i] = 0;
                }
            }
        }
        trace[k + 1] = sqrt(scdo_fro2(r, 1, N));
    }
    free(r);
    return capped;
}

/* ---------------------------------------------------------------- expansion (definition) */

/*
 * out[idx] = sum_{j<w} c[j] * prod_i s_{j,i}[idx_i], the terms added in the order j = 0..w-1
 * into one f64 accumulator per entry.  With order = 2 this is S_w C_w T_w^T.
 */
void scdo_expand(int order, const int64_t* dims, int64_t w, const uint64_t* const* signs,
                 const double* c, double* out)
{
    int64_t idx[SCDO_MAX_ORDER] = {0};
    int64_t N = total_size(order, dims);
    int64_t nw[SCDO_MAX_ORDER];
    for (int i = 0; i < order; ++i) nw[i] = words_for(dims[i]);
    if (N == 0) return;
    int64_t pos = 0;
    do {
        double acc = 0.0;
        for (int64_t j = 0; j < w; ++j) {
            double sg = 1.0;
            for (int i = 0; i < order; ++i) sg *= sign_at(signs[i] + j * nw[i], idx[i]);
            acc += c[j] * sg;
        }
        out[pos] = acc;
        ++pos;
    } while (next_index(order, dims, idx));
}

/* ---------------------------------------------------------------- product with a vector (Section 6.1) */

/*
 * y = (sum_{j<w} c_j s_j t_j^T) x          (transpose == 0:  x has n entries, y has m)
 * y = (sum_{j<w} c_j s_j t_j^T)^T x        (transpose != 0:  x has m entries, y has n)
 * straight from the factors: z_j = c_j <t_j, x>, then y = sum_j z_j s_j with the terms added in
 * the order j = 0..w-1 (for the transpose the two sign vectors trade places).
 */
void scdo_apply(int64_t m, int64_t n, int64_t w, const uint64_t* S, const uint64_t* T, const double* c,
                int transpose, const double* x, double* y)
{
    const uint64_t* in_bits = transpose ? S : T;
    const uint64_t* out_bits = transpose ? T : S;
    int64_t nin = transpose ? m : n, nout = transpose ? n : m;
    int64_t win = words_for(nin), wout = words_for(nout);
    for (int64_t i = 0; i < nout; ++i) y[i] = 0.0;
    for (int64_t j = 0; j < w; ++j) {
        double z = 0.0;
        for (int64_t l = 0; l < nin; ++l) z += sign_at(in_bits + j * win, l) * x[l];
        z *= c[j];
        for (int64_t i = 0; i < nout; ++i) y[i] += sign_at(out_bits + j * wout, i) * z;
    }
}

/* ---------------------------------------------------------------- brute force (Section 2.2, 3.1) */

/* ||A||_signed-cut = max over s in {-1,1}^m of ||A^T s||_1 (LeftSgnCut), by enumeration. m <= 24. */
double scdo_bruteforce_signed_cut_norm(const double* A, int64_t m, int64_t n, uint64_t* best_s)
{
    double best = -INFINITY;
    uint64_t arg = 0;
    if (m > 24) return NAN;
    for (uint64_t mask = 0; mask < (1ull << m); ++mask) {
        double tot = 0.0;
        for (int64_t l = 0; l < n; ++l) {
            double col = 0.0;
            for (int64_t i = 0; i < m; ++i) col += ((mask >> i) & 1ull) ? -A[i * n + l] : A[i * n + l];
            tot += fabs(col);
        }
        if (tot > best) {
            best = tot;
            arg = mask;
        }
    }
    if (best_s) *best_s = arg;
    return best;
}
