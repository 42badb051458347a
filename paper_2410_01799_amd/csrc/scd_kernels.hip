// HIP kernels of libscd for gfx950 (wave64).  Everything here is memory-bound sign-flip-and-add
// work (Section 3.4 of arXiv 2410.01799: no multiplies are needed), so there is no MFMA code.
//
//  rowpass  : one pass over a rows x cols array X with a sign vector t over the columns:
//             u = X t, s = sgn(u) and, in the same pass, the per-workgroup partial sums of
//             s^T X (Algorithm 4 lines 5 and 6 read the matrix once instead of twice).  On the
//             remainder itself it can first subtract the finished term (Algorithm 5 line 10) and
//             sum the squares for ||R||_F.
//  reduce   : fixed-order sum of the partials -> R^T s, t = sgn(.), c = sum |.| (Algorithm 4 line 7
//             via Section 3.1: <s, R t> = ||R^T s||_1), packs s from u with 64-lane ballots.
//  kron     : Kronecker products of sign bitsets for the tensor sweep (Algorithm 12 lines 5-7).
//  expand   : the definition sum_j c_j s_j t_j^T with one f64 accumulator per entry.
#include <stddef.h>

#include "scd_device.h"
#include "scd_rng.h"

namespace scd {

// ------------------------------------------------------------------------------------------------
// small device helpers

__device__ __forceinline__ uint32_t bit_at(const uint64_t* b, int64_t i)
{
    return (uint32_t)((b[i >> 6] >> (i & 63)) & 1ull);
}

__device__ __forceinline__ float flip(float x, uint32_t neg)
{
    return __uint_as_float(__float_as_uint(x) ^ (neg << 31));
}
__device__ __forceinline__ double flip(double x, uint32_t neg)
{
    return __longlong_as_double(__double_as_longlong(x) ^ ((long long)neg << 63));
}

// Workgroup barrier for LDS exchange only.  __syncthreads() would also wait for every outstanding
// global load, i.e. for the rows being prefetched for the next batch; this waits for LDS alone.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Sum over the 64 lanes by an xor butterfly.  a+b and b+a round alike, so every lane ends with
// the same bits, and the order of additions is fixed: results do not depend on timing.
__device__ __forceinline__ double wave_sum(double a)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, kWave);
    return a;
}

// Fixed-order sum of x[0..n) by one full wave; every lane returns the same value.
__device__ __forceinline__ double sum_fixed(const double* x, int n)
{
    double a = 0.0;
    for (int i = threadIdx.x & (kWave - 1); i < n; i += kWave) a += x[i];
    return wave_sum(a);
}

// ------------------------------------------------------------------------------------------------
// row pass, generic form: any rows, cols; two phases inside a workgroup.
//   phase A  one wave per row: optional update, squares, signed row sum, sign of the row
//   phase B  one thread per column: signed sum of the workgroup's rows (re-read from cache)

template <typename TE>
__device__ void rowpass_generic_body(TE* __restrict__ X, int64_t rows, int64_t cols, int rows_per_wg,
                                     bool do_update, bool do_norm, bool do_rows, bool do_cols,
                                     const uint64_t* __restrict__ sumbits, const uint64_t* __restrict__ updbits,
                                     const uint64_t* __restrict__ rowbits, TE ck, TE* __restrict__ partials,
                                     double* __restrict__ u, double* __restrict__ fparts, uint8_t* sh_s,
                                     double* sh_red)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_wg;
    const int64_t r1 = (r0 + rows_per_wg < rows) ? r0 + rows_per_wg : rows;
    double fsq = 0.0;

    for (int64_t r = r0 + wv; r < r1; r += kWavesPerBlock) {
        TE* row = X + r * cols;
        uint32_t sold = (do_update || !do_rows) ? bit_at(rowbits, r) : 0u;
        TE p = 0;
        double f = 0.0;
        if (do_update || do_norm || do_rows) {
            for (int64_t l = lane; l < cols; l += kWave) {
                TE x = row[l];
                if (do_update) {
                    // x - ck * s_r * t_l : the product of the signs picks +ck or -ck
                    uint32_t neg = sold ^ bit_at(updbits, l);
                    x = x - flip(ck, neg);
                    row[l] = x;
                }
                if (do_norm) f += (double)x * (double)x;
                if (do_rows) p += flip(x, bit_at(sumbits, l));
            }
        }
        fsq += f;
        if (do_rows) {
            double ur = wave_sum((double)p);
            if (lane == 0) {
                u[r] = ur;
                sh_s[r - r0] = (ur < 0.0) ? 1 : 0;
            }
        } else if (lane == 0) {
            sh_s[r - r0] = (uint8_t)sold;
        }
    }
    if (do_norm) {
        fsq = wave_sum(fsq);
        if (lane == 0) sh_red[wv] = fsq;
    }
    __syncthreads();
    if (do_norm && threadIdx.x == 0) {
        double t = 0.0;
        for (int i = 0; i < kWavesPerBlock; ++i) t += sh_red[i];
        fparts[blockIdx.x] = t;
    }
    if (do_cols) {
        const int nr = (int)(r1 - r0);
        for (int64_t l = threadIdx.x; l < cols; l += kBlock) {
            TE acc = 0;
            const TE* colp = X + r0 * cols + l;
            for (int r = 0; r < nr; ++r) acc += flip(colp[(int64_t)r * cols], (uint32_t)sh_s[r]);
            partials[(int64_t)blockIdx.x * cols + l] = acc;
        }
    }
}

// The fields of the device state a row pass needs, read one by one: a whole-struct copy would be
// placed in LDS or scratch by the compiler and serialise the loads behind it.
struct StateView {
    int64_t k;
    double c_prev;
    int32_t j, done, t0_given, max_iters, active, sweep_rng;
};

__device__ __forceinline__ StateView view_state(const State* s)
{
    StateView v;
    v.k = s->k;
    v.c_prev = s->c_prev;
    v.j = s->j;
    v.done = s->done;
    v.t0_given = s->t0_given;
    v.max_iters = s->max_iters;
    v.active = s->active;
    v.sweep_rng = s->sweep_rng;
    return v;
}

// What the level-0 pass of this sweep has to do, decided alike by every workgroup (Algorithm 4
// line 8: stop when c_j <= c_{j-1}).  Returns false when the sweep is to be skipped.
struct Decision {
    int mode;
    double c;
    double ck;
};

__device__ __forceinline__ bool decide_level0(const RowPassArgs& a, const StateView& st, double c, Decision& d)
{
    d.c = 0.0;
    d.ck = 0.0;
    d.mode = PASS_START;
    if (st.done) return false;
    if (st.j == 0) return true;
    d.c = c;  // sum of the partial sums of |R^T s|, the same bits in every workgroup
    bool conv = (d.c <= st.c_prev) || (st.j >= st.max_iters);
    d.mode = conv ? PASS_UPDATE : PASS_CONT;
    d.ck = d.c / a.total;
    return true;
}

// Bookkeeping of the level-0 pass, done after the pass itself: append the finished term and write
// the state the rest of the sweep reads.  Called by every thread of every workgroup; the sign copy
// is spread over all of them, the state is written by one thread, field by field.
template <typename TE>
__device__ __forceinline__ void level0_bookkeeping(const RowPassArgs& a, const StateView& st, const Decision& d)
{
    if (d.mode == PASS_UPDATE) {
        // S_{k+1} = [S_k s], T_{k+1} = [T_k t]  (Algorithm 5 lines 8-9): every workgroup copies a slice
        for (int i = 0; i < a.order; ++i) {
            uint64_t* dst = a.out_signs[i] + st.k * a.words[i];
            for (int p = blockIdx.x * kBlock + threadIdx.x; p < a.words[i]; p += gridDim.x * kBlock)
                dst[p] = a.cur_signs[i][p];
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        const State* cu = a.cur;
        State* nx = a.next;
        nx->w_target = cu->w_target;
        nx->max_iters = st.max_iters;
        nx->done = 0;
        nx->active = 1;
        nx->passes = cu->passes + 1;
        nx->c_last = d.c;
        nx->t0_given = 0;
        if (d.mode == PASS_START) {
            nx->k = st.k;
            nx->updates = cu->updates;
            nx->warn = cu->warn;
            nx->j = 1;
            nx->c_prev = -INFINITY;
            nx->norm_pending = 1;
            nx->sweep_rng = st.t0_given ? 0 : 1;
        } else if (d.mode == PASS_CONT) {
            nx->k = st.k;
            nx->updates = cu->updates;
            nx->warn = cu->warn;
            nx->j = st.j + 1;
            nx->c_prev = d.c;
            nx->norm_pending = 0;
            nx->sweep_rng = 0;
        } else {
            ((TE*)a.c_out)[st.k] = (TE)d.ck;  // c_{k+1} (Algorithm 5 line 7), normalised
            a.iters_out[st.k] = st.j;
            nx->warn = (d.c <= st.c_prev) ? cu->warn : 1;
            nx->k = st.k + 1;
            nx->updates = cu->updates + 1;
            nx->j = 1;
            nx->c_prev = -INFINITY;
            nx->norm_pending = 1;
            nx->sweep_rng = 1;
        }
    }
}

template <typename TE>
__global__ void __launch_bounds__(kBlock) rowpass_generic_kernel(RowPassArgs a)
{
    __shared__ uint8_t sh_s[kMaxRowsPerWg];
    __shared__ double sh_red[kWavesPerBlock];
    if (a.level == 0) {
        const StateView st = view_state(a.cur);
        Decision d;
        if (!decide_level0(a, st, sum_fixed(a.cparts, a.ncparts), d)) {
            if (blockIdx.x == 0 && threadIdx.x == 0) a.next->active = 0;
            return;
        }
        const bool upd = d.mode == PASS_UPDATE;
        const bool start = d.mode == PASS_START;
        const uint64_t* sumbits = (upd || (start && !st.t0_given)) ? a.sign_rng : a.sign_cur;
        rowpass_generic_body<TE>((TE*)a.X, a.rows, a.cols, a.rows_per_wg, upd, upd || start, true, true, sumbits,
                                 a.sign_cur, a.row_bits, (TE)d.ck, (TE*)a.partials, a.u, a.fparts, sh_s, sh_red);
        level0_bookkeeping<TE>(a, st, d);
    } else {
        const StateView st = view_state(a.next);
        if (!st.active) return;
        const uint64_t* sumbits = st.sweep_rng ? a.sign_rng : a.sign_cur;
        rowpass_generic_body<TE>((TE*)a.X, a.rows, a.cols, a.rows_per_wg, false, false, true, true, sumbits,
                                 a.sign_cur, a.row_bits, (TE)0, (TE*)a.partials, a.u, a.fparts, sh_s, sh_red);
    }
}

// Half steps on caller data (no state): rows only, or columns only with s given in `rowbits`.
template <typename TE>
__global__ void __launch_bounds__(kBlock)
    halfstep_kernel(TE* X, int64_t rows, int64_t cols, int rows_per_wg, int do_rows, const uint64_t* sumbits,
                    const uint64_t* rowbits, TE* partials, double* u)
{
    __shared__ uint8_t sh_s[kMaxRowsPerWg];
    __shared__ double sh_red[kWavesPerBlock];
    rowpass_generic_body<TE>(X, rows, cols, rows_per_wg, false, false, do_rows != 0, do_rows == 0, sumbits, nullptr,
                             rowbits, (TE)0, partials, u, nullptr, sh_s, sh_red);
}

// ------------------------------------------------------------------------------------------------
// row pass, register-tiled form for rows of at most 64 KB whose length is a multiple of 16 bytes.
//
// The 256 threads of a workgroup share each row: thread t owns the 16-byte chunks t, t+256, ...
// (CPT of them), so one wave reads 1 KB contiguous per chunk index.  RB rows are in registers at a
// time and the next RB rows are already being loaded while these are reduced.  Because a thread
// keeps its own columns for every row, the column partial sums never leave its registers until
// the workgroup is done: the matrix is read exactly once per alternation.
//
// Loads are never predicated: a row or chunk index past the end is clamped to the last valid one
// (the address stays in bounds) and the value is zeroed afterwards, only in the code path that
// handles a ragged batch.  Full batches run without any select.

template <typename TE>
struct Vec16;
template <>
struct Vec16<float> {
    typedef float4 type;
    static constexpr int N = 4;
};
template <>
struct Vec16<double> {
    typedef double2 type;
    static constexpr int N = 2;
};

template <typename TE, int CPT, int RB>
struct Tile {
    static constexpr int VE = Vec16<TE>::N;
    TE x[RB][CPT * VE];
    uint32_t rowsign;  // bit r: current sign of row rb+r (read by the update)
};

template <typename TE, int CPT, int RB>
__device__ __forceinline__ void tile_load(Tile<TE, CPT, RB>& t, const TE* __restrict__ X, int64_t cols, int64_t rb,
                                          int64_t r1, int64_t nch, const uint64_t* __restrict__ rowbits, int64_t rows,
                                          bool valid)
{
    // Never predicated and never behind a branch: a conditional prefetch would make the compiler
    // wait for it at the next join.  A batch that does not exist (`valid` false) is loaded from one
    // 16-byte location instead, a broadcast that costs next to nothing and is never used.
    constexpr int VE = Vec16<TE>::N;
    typedef typename Vec16<TE>::type V;
    {
        const int64_t wlast = (rows - 1) >> 6;
        int64_t w0i = rb >> 6;
        w0i = w0i < wlast ? w0i : wlast;
        const int64_t w1i = w0i < wlast ? w0i + 1 : wlast;
        const uint64_t w0 = rowbits[w0i], w1 = rowbits[w1i];
        const int sh = (int)(rb & 63);
        t.rowsign = (uint32_t)((w0 >> sh) | (sh ? (w1 << (64 - sh)) : 0ull));
    }
    int64_t chs[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int64_t ch = threadIdx.x + c * kBlock;
        const int64_t chc = ch < nch ? ch : nch - 1;
        chs[c] = valid ? chc : 0;
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        int64_t row = rb + r;
        row = row < r1 ? row : r1 - 1;
        const V* rowp = (const V*)(X + row * cols);
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const V v = rowp[chs[c]];
            if constexpr (VE == 4) {
                t.x[r][c * 4 + 0] = v.x;
                t.x[r][c * 4 + 1] = v.y;
                t.x[r][c * 4 + 2] = v.z;
                t.x[r][c * 4 + 3] = v.w;
            } else {
                t.x[r][c * 2 + 0] = v.x;
                t.x[r][c * 2 + 1] = v.y;
            }
        }
    }
}

// Sign bits of this thread's columns, element e of chunk c in bit c*VE+e (0 past the end).
template <typename TE, int CPT>
__device__ __forceinline__ uint64_t gather_bits(const uint64_t* __restrict__ bits, int64_t nch)
{
    constexpr int VE = Vec16<TE>::N;
    uint64_t out = 0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int64_t ch = threadIdx.x + c * kBlock;
        const int64_t chc = ch < nch ? ch : nch - 1;
        const int64_t col = chc * VE;  // VE divides 64: a chunk never straddles a word
        const uint64_t w = bits[col >> 6];
        const uint64_t b = (w >> (col & 63)) & ((1ull << VE) - 1);
        out |= (ch < nch ? b : 0ull) << (c * VE);
    }
    return out;
}

// One batch of RB rows.  FULL: every row of the batch and every chunk of this thread exists.
template <typename TE, int CPT, int RB, bool UPD, bool FULL>
__device__ __forceinline__ void tile_process(Tile<TE, CPT, RB>& t, TE* __restrict__ X, int64_t cols, int64_t rb,
                                             int64_t r1, int64_t nch, uint64_t sumb, uint64_t updb, TE ck, TE* acc,
                                             double& fsq, double* __restrict__ u,
                                             double (*sh_u)[kWavesPerBlock][RB], int parity)
{
    constexpr int VE = Vec16<TE>::N;
    constexpr int NE = CPT * VE;
    typedef typename Vec16<TE>::type V;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    double ps[RB];
    if constexpr (!FULL) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const bool rok = rb + r < r1;
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const bool ok = rok && (threadIdx.x + c * kBlock < nch);
#pragma unroll
                for (int e = 0; e < VE; ++e) t.x[r][c * VE + e] = ok ? t.x[r][c * VE + e] : (TE)0;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        if constexpr (UPD) {
            // R <- R - ck s t^T (Algorithm 5 line 10), and the squares of the new remainder
            const bool rok = FULL || (rb + r < r1);
            const int64_t rowc = rok ? rb + r : r1 - 1;
            const uint32_t sold = (t.rowsign >> r) & 1u;
#pragma unroll
            for (int e = 0; e < NE; ++e) {
                const uint32_t neg = sold ^ (uint32_t)((updb >> e) & 1ull);
                t.x[r][e] = t.x[r][e] - flip(ck, neg);
            }
            V* rowp = (V*)(X + rowc * cols);
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                V v;
                if constexpr (VE == 4) v = V{t.x[r][c * 4], t.x[r][c * 4 + 1], t.x[r][c * 4 + 2], t.x[r][c * 4 + 3]};
                else v = V{t.x[r][c * 2], t.x[r][c * 2 + 1]};
                if constexpr (FULL) {
                    rowp[threadIdx.x + c * kBlock] = v;
                } else {
                    const bool ok = rok && (threadIdx.x + c * kBlock < nch);
                    if (ok) rowp[threadIdx.x + c * kBlock] = v;
                    else {
#pragma unroll
                        for (int e = 0; e < VE; ++e) t.x[r][c * VE + e] = 0;  // padding stays zero
                    }
                }
            }
            // squares in f64: large entries must not overflow, small ones must not vanish
#pragma unroll
            for (int e = 0; e < NE; ++e) fsq += (double)t.x[r][e] * (double)t.x[r][e];
        }
        TE p = 0;
#pragma unroll
        for (int e = 0; e < NE; ++e) p += flip(t.x[r][e], (uint32_t)((sumb >> e) & 1ull));
        ps[r] = (double)p;
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) ps[r] = wave_sum(ps[r]);
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) sh_u[parity][wv][r] = ps[r];
    }
    lds_barrier();
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        double ur = 0.0;
#pragma unroll
        for (int q = 0; q < kWavesPerBlock; ++q) ur += sh_u[parity][q][r];
        if (threadIdx.x == r && (FULL || rb + r < r1)) u[rb + r] = ur;
        const uint32_t neg = ur < 0.0 ? 1u : 0u;
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[e] += flip(t.x[r][e], neg);
    }
}

template <typename TE, int CPT, int RB, bool UPD>
__device__ __forceinline__ void tile_step(Tile<TE, CPT, RB>& t, TE* __restrict__ X, int64_t cols, int64_t rb,
                                          int64_t r1, int64_t nch, bool full_cols, uint64_t sumb, uint64_t updb, TE ck,
                                          TE* acc, double& fsq, double* __restrict__ u,
                                          double (*sh_u)[kWavesPerBlock][RB], int parity)
{
    if (full_cols && rb + RB <= r1)
        tile_process<TE, CPT, RB, UPD, true>(t, X, cols, rb, r1, nch, sumb, updb, ck, acc, fsq, u, sh_u, parity);
    else
        tile_process<TE, CPT, RB, UPD, false>(t, X, cols, rb, r1, nch, sumb, updb, ck, acc, fsq, u, sh_u, parity);
}

// `ta` already holds the first batch (its loads were issued before the pass was decided).
template <typename TE, int CPT, int RB, bool UPD>
__device__ __forceinline__ void rowpass_tiled_body(Tile<TE, CPT, RB>& ta, TE* __restrict__ X, int64_t rows,
                                                   int64_t cols, int64_t r0, int64_t r1, uint64_t sumb, uint64_t updb,
                                                   const uint64_t* __restrict__ rowbits, TE ck,
                                                   TE* __restrict__ partials, double* __restrict__ u,
                                                   double* __restrict__ fparts)
{
    constexpr int VE = Vec16<TE>::N;
    constexpr int NE = CPT * VE;
    typedef typename Vec16<TE>::type V;
    __shared__ double sh_u[2][kWavesPerBlock][RB];
    __shared__ double sh_f[kWavesPerBlock];
    const int64_t nch = cols / VE;
    const bool full_cols = nch == (int64_t)CPT * kBlock;
    TE acc[NE];
#pragma unroll
    for (int e = 0; e < NE; ++e) acc[e] = 0;
    double fsq = 0.0;

    // Two register tiles alternate: while one batch is reduced, the loads of the next one are in
    // flight.  Inside the loop every load is unconditional (see tile_load).
    Tile<TE, CPT, RB> tb;
    const int64_t nb = (r1 - r0 + RB - 1) / RB;
    int64_t b = 0;
    for (; b + 1 < nb; b += 2) {
        const int64_t rb = r0 + b * RB;
        tile_load<TE, CPT, RB>(tb, X, cols, rb + RB, r1, nch, rowbits, rows, true);
        tile_step<TE, CPT, RB, UPD>(ta, X, cols, rb, r1, nch, full_cols, sumb, updb, ck, acc, fsq, u, sh_u, 0);
        tile_load<TE, CPT, RB>(ta, X, cols, rb + 2 * RB, r1, nch, rowbits, rows, b + 2 < nb);
        tile_step<TE, CPT, RB, UPD>(tb, X, cols, rb + RB, r1, nch, full_cols, sumb, updb, ck, acc, fsq, u, sh_u, 1);
    }
    if (b < nb)
        tile_step<TE, CPT, RB, UPD>(ta, X, cols, r0 + b * RB, r1, nch, full_cols, sumb, updb, ck, acc, fsq, u, sh_u, 0);
    V* pp = (V*)(partials + (int64_t)blockIdx.x * cols);
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int64_t ch = threadIdx.x + c * kBlock;
        if (ch < nch) {
            V v;
            if constexpr (VE == 4) v = V{acc[c * 4], acc[c * 4 + 1], acc[c * 4 + 2], acc[c * 4 + 3]};
            else v = V{acc[c * 2], acc[c * 2 + 1]};
            pp[ch] = v;
        }
    }
    if constexpr (UPD) {
        fsq = wave_sum(fsq);
        if ((threadIdx.x & (kWave - 1)) == 0) sh_f[threadIdx.x / kWave] = fsq;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int i = 0; i < kWavesPerBlock; ++i) t += sh_f[i];
            fparts[blockIdx.x] = t;
        }
    }
}

template <typename TE, int CPT, int RB>
__global__ void __launch_bounds__(kBlock) rowpass_tiled_kernel(RowPassArgs a)
{
    constexpr int VE = Vec16<TE>::N;
    const int64_t r0 = (int64_t)blockIdx.x * a.rows_per_wg;
    const int64_t r1 = (r0 + a.rows_per_wg < a.rows) ? r0 + a.rows_per_wg : a.rows;
    const int64_t nch = a.cols / VE;
    // Nothing read here depends on what this pass turns out to be: start the loads of the first
    // rows, of both sign vectors, of the state and of the partial sums of c together, so that
    // their latencies overlap instead of adding up.
    Tile<TE, CPT, RB> ta;
    tile_load<TE, CPT, RB>(ta, (const TE*)a.X, a.cols, r0, r1, nch, a.row_bits, a.rows, true);
    const StateView st = view_state(a.level == 0 ? a.cur : a.next);
    double cp = 0.0;
    if (a.level == 0)
        for (int i = threadIdx.x & (kWave - 1); i < a.ncparts; i += kWave) cp += a.cparts[i];
    const uint64_t bcur = gather_bits<TE, CPT>(a.sign_cur, nch);
    const uint64_t brng = gather_bits<TE, CPT>(a.sign_rng, nch);
    if (a.level == 0) {
        Decision d;
        if (!decide_level0(a, st, wave_sum(cp), d)) {
            if (blockIdx.x == 0 && threadIdx.x == 0) a.next->active = 0;
            return;
        }
        if (d.mode == PASS_CONT) {
            rowpass_tiled_body<TE, CPT, RB, false>(ta, (TE*)a.X, a.rows, a.cols, r0, r1, bcur, 0ull, a.row_bits, (TE)0,
                                                   (TE*)a.partials, a.u, a.fparts);
        } else {
            // a start pass is an update by zero: the remainder is rewritten unchanged and its squares summed
            const bool upd = d.mode == PASS_UPDATE;
            const uint64_t sumb = (upd || !st.t0_given) ? brng : bcur;
            rowpass_tiled_body<TE, CPT, RB, true>(ta, (TE*)a.X, a.rows, a.cols, r0, r1, sumb, bcur, a.row_bits,
                                                  upd ? (TE)d.ck : (TE)0, (TE*)a.partials, a.u, a.fparts);
        }
        level0_bookkeeping<TE>(a, st, d);
    } else {
        if (!st.active) return;
        rowpass_tiled_body<TE, CPT, RB, false>(ta, (TE*)a.X, a.rows, a.cols, r0, r1, st.sweep_rng ? brng : bcur, 0ull,
                                               a.row_bits, (TE)0, (TE*)a.partials, a.u, a.fparts);
    }
}

// ------------------------------------------------------------------------------------------------
// reduce: W[l] = sum over the partial rows, in f64 and in a fixed order.  One block of 16 waves per
// 64 columns; wave q adds the partial rows q, q+16, ... (16 independent loads in flight at a time),
// then wave 0 adds the 16 wave sums in order.

constexpr int kRedWaves = 16;
constexpr int kRedBlock = kRedWaves * kWave;

template <typename TA>
__device__ __forceinline__ double column_sum(const TA* __restrict__ P, int nparts, int64_t cols, int64_t col,
                                             double (*sh)[kWave])
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    double s = 0.0;
    if (col < cols) {
        const TA* base = P + col;
        int p = wv;
        for (; p + 15 * kRedWaves < nparts; p += 16 * kRedWaves) {
            TA tmp[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) tmp[i] = base[(int64_t)(p + i * kRedWaves) * cols];
#pragma unroll
            for (int i = 0; i < 16; ++i) s += (double)tmp[i];
        }
        for (; p < nparts; p += kRedWaves) s += (double)base[(int64_t)p * cols];
    }
    sh[wv][lane] = s;
    __syncthreads();
    double v = 0.0;
    if (wv == 0) {
#pragma unroll
        for (int q = 0; q < kRedWaves; ++q) v += sh[q][lane];
    }
    return v;
}

template <typename TA>
__global__ void __launch_bounds__(kRedBlock) reduce_kernel(ReduceArgs a)
{
    __shared__ double sh[kRedWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int64_t col = (int64_t)blockIdx.x * kWave + lane;
    const int64_t rwords = (a.rows + 63) / 64;
    // Everything this block reads is independent of the state: start all loads, then look at it.
    // (An inactive sweep reads valid, stale data and writes nothing.)
    const State* sp = a.next;
    const int32_t active = sp->active, norm_pending = sp->norm_pending;
    const int64_t k = sp->k, w_target = sp->w_target;
    const int64_t wd0 = (int64_t)blockIdx.x * kRedWaves + wv;
    const int64_t i0 = wd0 * 64 + lane;
    const double u0 = (wd0 < rwords && i0 < a.rows) ? a.u[i0] : 0.0;
    double fp = 0.0;
    if (a.final && blockIdx.x == 0 && wv == 1)
        for (int i = lane; i < a.nfparts; i += kWave) fp += a.fparts[i];
    const double v = column_sum<TA>((const TA*)a.partials, a.nparts, a.cols, col, sh);
    if (!active) return;
    if (wv == 0) {
        if (col < a.cols) a.W[col] = v;
        if (a.final) {
            // t = sgn(R^T s) packed from the ballot; c = sum |R^T s| (Algorithm 4 lines 6-7)
            const uint64_t word = __ballot(col < a.cols && v < 0.0);
            const double cabs = wave_sum(col < a.cols ? fabs(v) : 0.0);
            if (lane == 0) {
                a.last_bits[blockIdx.x] = word;
                a.cparts[blockIdx.x] = cabs;
            }
        }
    }
    // s = sgn(u) for this level's mode, one word per wave-ballot
    if (wd0 < rwords) {
        const uint64_t word = __ballot(i0 < a.rows && u0 < 0.0);
        if (lane == 0) a.row_bits[wd0] = word;
    }
    for (int64_t wd = wd0 + (int64_t)gridDim.x * kRedWaves; wd < rwords; wd += (int64_t)gridDim.x * kRedWaves) {
        const int64_t i = wd * 64 + lane;
        const uint64_t word = __ballot(i < a.rows && a.u[i] < 0.0);
        if (lane == 0) a.row_bits[wd] = word;
    }
    if (a.final) {
        // random start of the term after the current one, last mode (Algorithm 4 line 2)
        const int64_t cwords = (a.cols + 63) / 64;
        for (int64_t wd = (int64_t)blockIdx.x * kRedBlock + threadIdx.x; wd < cwords; wd += (int64_t)gridDim.x * kRedBlock)
            a.rng_last[wd] = rng_word_masked(a.seed, (uint64_t)k + 1, (uint32_t)a.last_mode, wd, a.cols);
        if (blockIdx.x == 0 && wv == 1) {
            const double F = wave_sum(fp);
            if (lane == 0 && norm_pending) a.trace[k] = sqrt(F);
            // cur <- next, word by word, with `done` set once the requested width is reached
            constexpr int kWords = (int)(sizeof(State) / 4);
            constexpr int kDoneWord = (int)(offsetof(State, done) / 4);
            static_assert(sizeof(State) % 4 == 0 && kWords <= kWave, "state is copied by one wave");
            if (lane < kWords) {
                uint32_t wv32 = ((const uint32_t*)a.next)[lane];
                if (lane == kDoneWord) wv32 = (k >= w_target) ? 1u : 0u;
                ((uint32_t*)a.cur)[lane] = wv32;
            }
        }
    }
}

// Column half step on caller data: same reduction without any state.
template <typename TA>
__global__ void __launch_bounds__(kRedBlock)
    reduce_plain_kernel(const TA* P, int nparts, int64_t cols, double* W, uint64_t* bits, double* cparts)
{
    __shared__ double sh[kRedWaves][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = threadIdx.x / kWave;
    const int64_t col = (int64_t)blockIdx.x * kWave + lane;
    const double v = column_sum<TA>(P, nparts, cols, col, sh);
    if (wv == 0) {
        if (col < cols && W) W[col] = v;
        const uint64_t word = __ballot(col < cols && v < 0.0);
        const double cabs = wave_sum(col < cols ? fabs(v) : 0.0);
        if (lane == 0) {
            if (bits) bits[blockIdx.x] = word;
            cparts[blockIdx.x] = cabs;
        }
    }
}

__global__ void sum_parts_kernel(const double* parts, int n, double* out)
{
    double s = sum_fixed(parts, n);
    if (threadIdx.x == 0) *out = s;
}

// ------------------------------------------------------------------------------------------------
// Kronecker sign vectors for tensors of order >= 3 (Algorithm 12 lines 5-7): for level l the bit of
// column q is the xor of the sign bits of modes l+1.. at the multi-index of q (last mode fastest).

__global__ void __launch_bounds__(kBlock) kron_kernel(KronArgs a)
{
    if (!a.force && !a.next->active) return;
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t term = (uint64_t)a.cur->k + (uint64_t)a.term_offset;
    int64_t wd = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave;  // one wave per output word
    const int64_t wstride = (int64_t)gridDim.x * kWavesPerBlock;
    int64_t total_words = 0;
    for (int l = 0; l + 2 < a.order; ++l) total_words += (a.cols[l] + 63) / 64;
    for (; wd < total_words; wd += wstride) {
        int l = 0;
        int64_t base = 0;
        while (l + 3 < a.order && wd >= base + (a.cols[l] + 63) / 64) {
            base += (a.cols[l] + 63) / 64;
            ++l;
        }
        int64_t q = (wd - base) * 64 + lane;
        const bool ok = q < a.cols[l];
        uint32_t bc = 0, br = 0;
        if (ok) {
            int64_t rest = q;
            for (int i = a.order - 1; i > l; --i) {
                const int64_t idx = rest % a.dims[i];
                rest /= a.dims[i];
                bc ^= bit_at(a.cur_signs[i], idx);
                br ^= (uint32_t)((rng_word(a.seed, term, (uint32_t)i, (uint64_t)(idx >> 6)) >> (idx & 63)) & 1ull);
            }
        }
        const uint64_t wc = __ballot(ok && bc);
        const uint64_t wr = __ballot(ok && br);
        if (lane == 0) {
            a.kron_cur[l][wd - base] = wc;
            a.kron_rng[l][wd - base] = wr;
        }
    }
    if (a.with_last) {
        const int last = a.order - 1;
        const int64_t cwords = (a.dims[last] + 63) / 64;
        for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < cwords; p += (int64_t)gridDim.x * kBlock)
            a.rng_last[p] = rng_word_masked(a.seed, term, (uint32_t)last, p, a.dims[last]);
    }
}

// Kronecker bitsets of modes 1.. for every term (used by expand for order >= 3):
// out[j][q] = xor_i>=1 signs[i][j][idx_i(q)].
struct KronTermsArgs {
    int32_t order;
    int64_t dims[SCD_MAX_ORDER];
    const uint64_t* signs[SCD_MAX_ORDER];
    int64_t w, cols;
    uint64_t* out;
};

__global__ void __launch_bounds__(kBlock) kron_terms_kernel(KronTermsArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t cw = (a.cols + 63) / 64;
    const int64_t total = a.w * cw;
    for (int64_t wd = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave; wd < total;
         wd += (int64_t)gridDim.x * kWavesPerBlock) {
        const int64_t j = wd / cw;
        const int64_t q = (wd % cw) * 64 + lane;
        uint32_t b = 0;
        const bool ok = q < a.cols;
        if (ok) {
            int64_t rest = q;
            for (int i = a.order - 1; i >= 1; --i) {
                const int64_t idx = rest % a.dims[i];
                rest /= a.dims[i];
                b ^= bit_at(a.signs[i] + j * ((a.dims[i] + 63) / 64), idx);
            }
        }
        const uint64_t word = __ballot(ok && b);
        if (lane == 0) a.out[wd] = word;
    }
}

// ------------------------------------------------------------------------------------------------
// expand: out[i][l] = sum_j c_j s_j[i] t_j[l], terms added in order into an f64 accumulator.
// A wave owns 64 columns (one word of t_j) and 32 rows (half a word of s_j).

constexpr int kExpRows = 32;

template <typename TE>
__global__ void __launch_bounds__(kBlock)
    expand_kernel(const uint64_t* __restrict__ S, const uint64_t* __restrict__ T, const TE* __restrict__ c, int64_t m,
                  int64_t n, int64_t w, TE* __restrict__ out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t cw = blockIdx.x;                                             // column word
    const int64_t rt = (int64_t)blockIdx.y * kWavesPerBlock + wv;              // row tile of 32
    const int64_t row0 = rt * kExpRows;
    if (row0 >= m) return;
    const int64_t mw = (m + 63) / 64, nw = (n + 63) / 64;
    const int64_t sw = row0 >> 6;
    const int sh = (int)(row0 & 63);
    double acc[kExpRows];
#pragma unroll
    for (int r = 0; r < kExpRows; ++r) acc[r] = 0.0;
    for (int64_t j = 0; j < w; ++j) {
        const uint64_t tw = T[j * nw + cw];
        const uint32_t sbits = (uint32_t)(S[j * mw + sw] >> sh);
        const double cj = (double)c[j];
        const double cl = flip(cj, (uint32_t)((tw >> lane) & 1ull));
#pragma unroll
        for (int r = 0; r < kExpRows; ++r) acc[r] += flip(cl, (sbits >> r) & 1u);
    }
    const int64_t col = cw * 64 + lane;
    if (col < n) {
#pragma unroll
        for (int r = 0; r < kExpRows; ++r)
            if (row0 + r < m) out[(row0 + r) * n + col] = (TE)acc[r];
    }
}

// ------------------------------------------------------------------------------------------------
// bitset utilities (Section 3.1)

template <typename TE>
__global__ void __launch_bounds__(kBlock) pack_kernel(const TE* x, int64_t n, uint64_t* bits)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t words = (n + 63) / 64;
    for (int64_t wd = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / kWave; wd < words;
         wd += (int64_t)gridDim.x * kWavesPerBlock) {
        const int64_t i = wd * 64 + lane;
        const uint64_t word = __ballot(i < n && x[i] < (TE)0);
        if (lane == 0) bits[wd] = word;
    }
}

template <typename TE>
__global__ void __launch_bounds__(kBlock) unpack_kernel(const uint64_t* bits, int64_t n, TE* x)
{
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (int64_t)gridDim.x * kBlock)
        x[i] = bit_at(bits, i) ? (TE)-1 : (TE)1;
}

__global__ void __launch_bounds__(kBlock) rng_kernel(uint64_t seed, uint64_t term, uint32_t mode, int64_t n,
                                                    uint64_t* bits)
{
    const int64_t words = (n + 63) / 64;
    for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < words; p += (int64_t)gridDim.x * kBlock)
        bits[p] = rng_word_masked(seed, term, mode, p, n);
}

// ------------------------------------------------------------------------------------------------
// plain streaming kernels: the measured ceiling the row pass is compared with, and the copy of
// known size that calibrates the memory counters.

__global__ void __launch_bounds__(kBlock) stream_read_kernel(const float4* __restrict__ x, int64_t n4, float* sink)
{
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    for (; i + 7 * stride < n4; i += 8 * stride) {
        float4 v[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) v[q] = x[i + q * stride];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            acc.x += v[q].x;
            acc.y += v[q].y;
            acc.z += v[q].z;
            acc.w += v[q].w;
        }
    }
    for (; i < n4; i += stride) {
        const float4 v = x[i];
        acc.x += v.x;
        acc.y += v.y;
        acc.z += v.z;
        acc.w += v.w;
    }
    if (acc.x + acc.y + acc.z + acc.w == 1.2345e38f) *sink = acc.x;  // keeps the loads alive
}

__global__ void __launch_bounds__(kBlock) stream_copy_kernel(const float4* __restrict__ x, float4* __restrict__ y, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n4; i += stride) y[i] = x[i];
}

hipError_t launch_stream_read(const void* x, int64_t bytes, int grid, float* sink, hipStream_t st)
{
    hipLaunchKernelGGL(stream_read_kernel, dim3(grid), dim3(kBlock), 0, st, (const float4*)x, bytes / 16, sink);
    return hipGetLastError();
}

hipError_t launch_stream_copy(const void* x, void* y, int64_t bytes, int grid, hipStream_t st)
{
    hipLaunchKernelGGL(stream_copy_kernel, dim3(grid), dim3(kBlock), 0, st, (const float4*)x, (float4*)y, bytes / 16);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------
// launchers

static int grid_for(int64_t items, int per_block, int cap)
{
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

bool fast_rowpass_supported(scd_dtype dt, int64_t cols, int level)
{
    (void)level;
    const int ve = dt == SCD_F32 ? 4 : 2;
    if (cols % ve) return false;
    const int64_t nch = cols / ve;
    const int64_t cpt = (nch + kBlock - 1) / kBlock;
    return cpt >= 1 && cpt <= 16;
}

template <typename TE, int CPT>
static void launch_tiled_rb(const RowPassArgs& a, int grid, hipStream_t st)
{
    constexpr int VE = Vec16<TE>::N;
    // rows per register buffer: about 64 VGPRs per buffer (two buffers are live)
    constexpr int kRegsPerRow = CPT * VE * (int)sizeof(TE) / 4;
    constexpr int RB = kRegsPerRow > 32 ? 1 : (kRegsPerRow > 16 ? 2 : (kRegsPerRow > 8 ? 4 : 8));
    hipLaunchKernelGGL((rowpass_tiled_kernel<TE, CPT, RB>), dim3(grid), dim3(kBlock), 0, st, a);
}

template <typename TE>
static bool launch_tiled(const RowPassArgs& a, int grid, hipStream_t st)
{
    constexpr int VE = Vec16<TE>::N;
    const int64_t nch = a.cols / VE;
    const int cpt = (int)((nch + kBlock - 1) / kBlock);
    switch (cpt) {
        case 1: launch_tiled_rb<TE, 1>(a, grid, st); return true;
        case 2: launch_tiled_rb<TE, 2>(a, grid, st); return true;
        case 3:
        case 4: launch_tiled_rb<TE, 4>(a, grid, st); return true;
        case 5:
        case 6: launch_tiled_rb<TE, 6>(a, grid, st); return true;
        case 7:
        case 8: launch_tiled_rb<TE, 8>(a, grid, st); return true;
        case 9:
        case 10: launch_tiled_rb<TE, 10>(a, grid, st); return true;
        case 11:
        case 12: launch_tiled_rb<TE, 12>(a, grid, st); return true;
        case 13:
        case 14: launch_tiled_rb<TE, 14>(a, grid, st); return true;
        case 15:
        case 16: launch_tiled_rb<TE, 16>(a, grid, st); return true;
        default: return false;
    }
}

hipError_t launch_rowpass(const RowPassArgs& a, scd_dtype dt, int grid, int variant, hipStream_t st)
{
    // level >= 1 arrays are f64 whatever the input dtype
    const bool f64 = (a.level > 0) || dt == SCD_F64;
    const scd_dtype eff = f64 ? SCD_F64 : SCD_F32;
    bool done = false;
    if (variant == 1 && fast_rowpass_supported(eff, a.cols, a.level))
        done = f64 ? launch_tiled<double>(a, grid, st) : launch_tiled<float>(a, grid, st);
    if (!done) {
        if (f64) hipLaunchKernelGGL((rowpass_generic_kernel<double>), dim3(grid), dim3(kBlock), 0, st, a);
        else hipLaunchKernelGGL((rowpass_generic_kernel<float>), dim3(grid), dim3(kBlock), 0, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_reduce(const ReduceArgs& a, bool f32_partials, hipStream_t st)
{
    const int grid = (int)((a.cols + kWave - 1) / kWave);
    if (f32_partials) hipLaunchKernelGGL((reduce_kernel<float>), dim3(grid), dim3(kRedBlock), 0, st, a);
    else hipLaunchKernelGGL((reduce_kernel<double>), dim3(grid), dim3(kRedBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_kron(const KronArgs& a, hipStream_t st)
{
    int64_t words = 0;
    for (int l = 0; l + 2 < a.order; ++l) words += (a.cols[l] + 63) / 64;
    const int grid = grid_for(words > 0 ? words : 1, kWavesPerBlock, 1024);
    hipLaunchKernelGGL(kron_kernel, dim3(grid), dim3(kBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_pack(const void* values, scd_dtype dt, int64_t n, uint64_t* bits, hipStream_t st)
{
    const int grid = grid_for((n + 63) / 64, kWavesPerBlock, 4096);
    if (dt == SCD_F32) hipLaunchKernelGGL((pack_kernel<float>), dim3(grid), dim3(kBlock), 0, st, (const float*)values, n, bits);
    else hipLaunchKernelGGL((pack_kernel<double>), dim3(grid), dim3(kBlock), 0, st, (const double*)values, n, bits);
    return hipGetLastError();
}

hipError_t launch_unpack(const uint64_t* bits, int64_t n, scd_dtype dt, void* values, hipStream_t st)
{
    const int grid = grid_for(n, kBlock, 4096);
    if (dt == SCD_F32) hipLaunchKernelGGL((unpack_kernel<float>), dim3(grid), dim3(kBlock), 0, st, bits, n, (float*)values);
    else hipLaunchKernelGGL((unpack_kernel<double>), dim3(grid), dim3(kBlock), 0, st, bits, n, (double*)values);
    return hipGetLastError();
}

hipError_t launch_rng(uint64_t seed, uint64_t term, uint32_t mode, int64_t n, uint64_t* bits, hipStream_t st)
{
    const int grid = grid_for((n + 63) / 64, kBlock, 1024);
    hipLaunchKernelGGL(rng_kernel, dim3(grid), dim3(kBlock), 0, st, seed, term, mode, n, bits);
    return hipGetLastError();
}

hipError_t launch_kron_terms(int order, const int64_t* dims, const uint64_t* const* signs, int64_t w, uint64_t* out,
                             int64_t cols, hipStream_t st)
{
    KronTermsArgs a;
    a.order = order;
    for (int i = 0; i < order; ++i) {
        a.dims[i] = dims[i];
        a.signs[i] = signs[i];
    }
    a.w = w;
    a.cols = cols;
    a.out = out;
    const int grid = grid_for(w * ((cols + 63) / 64), kWavesPerBlock, 8192);
    hipLaunchKernelGGL(kron_terms_kernel, dim3(grid), dim3(kBlock), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_expand(const uint64_t* S, const uint64_t* T, const void* c, scd_dtype dt, int64_t m, int64_t n,
                         int64_t w, void* out, hipStream_t st)
{
    const int64_t tiles = (m + kExpRows - 1) / kExpRows;
    dim3 grid((unsigned)((n + 63) / 64), (unsigned)((tiles + kWavesPerBlock - 1) / kWavesPerBlock));
    if (dt == SCD_F32)
        hipLaunchKernelGGL((expand_kernel<float>), grid, dim3(kBlock), 0, st, S, T, (const float*)c, m, n, w, (float*)out);
    else
        hipLaunchKernelGGL((expand_kernel<double>), grid, dim3(kBlock), 0, st, S, T, (const double*)c, m, n, w, (double*)out);
    return hipGetLastError();
}

hipError_t launch_halfstep(const void* R, scd_dtype dt, int64_t m, int64_t n, int rows_per_wg, int grid, int do_rows,
                           const uint64_t* sumbits, const uint64_t* rowbits, void* partials, double* u, hipStream_t st)
{
    if (dt == SCD_F32)
        hipLaunchKernelGGL((halfstep_kernel<float>), dim3(grid), dim3(kBlock), 0, st, (float*)R, m, n, rows_per_wg, do_rows,
                           sumbits, rowbits, (float*)partials, u);
    else
        hipLaunchKernelGGL((halfstep_kernel<double>), dim3(grid), dim3(kBlock), 0, st, (double*)R, m, n, rows_per_wg,
                           do_rows, sumbits, rowbits, (double*)partials, u);
    return hipGetLastError();
}

hipError_t launch_reduce_plain(const void* partials, scd_dtype dt, int nparts, int64_t cols, double* W, uint64_t* bits,
                               double* cparts, hipStream_t st)
{
    const int grid = (int)((cols + kWave - 1) / kWave);
    if (dt == SCD_F32)
        hipLaunchKernelGGL((reduce_plain_kernel<float>), dim3(grid), dim3(kRedBlock), 0, st, (const float*)partials, nparts, cols, W, bits, cparts);
    else
        hipLaunchKernelGGL((reduce_plain_kernel<double>), dim3(grid), dim3(kRedBlock), 0, st, (const double*)partials, nparts, cols, W, bits, cparts);
    return hipGetLastError();
}

hipError_t launch_sum_parts(const double* parts, int n, double* out, hipStream_t st)
{
    hipLaunchKernelGGL(sum_parts_kernel, dim3(1), dim3(kWave), 0, st, parts, n, out);
    return hipGetLastError();
}

}  // namespace scd
