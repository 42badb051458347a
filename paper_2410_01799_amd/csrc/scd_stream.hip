// Persistent streaming engine: Algorithm 4 inside Algorithm 5 as ONE launch that streams the remainder from
// memory once per alternation, for matrices of any size that the register-resident engine cannot hold.
//
// Workgroup g (512 threads, one per compute unit) owns a block of whole rows for the entire launch.
//   row pass    the 512 threads share each row (thread t owns the 16-byte chunks t, t+512, ...).  For a batch
//               of RB rows: signed row sums with the bits of t (u = R t, Algorithm 4 line 5; the signs enter as
//               +-1.0 factors of a fused multiply-add, which rounds exactly like the flip-and-add of Section
//               3.4 in one instruction), joined across lanes and waves in f64 in a fixed order -> s_i for the
//               batch, then +-row added into per-thread column accumulators that stay in registers: both
//               products of an alternation from one read of R.  The first rows of the block are kept in LDS for the whole
//               launch (they are read from memory once per launch, not once per alternation); the others are
//               streamed with a second register tile in flight.  On a converged term the same pass first
//               subtracts c_k s t^T (Algorithm 5 line 10) and sums the squares.
//   hop 1       every workgroup lays its partial column sums out in column order in LDS and publishes them as
//               tagged 8-byte words, every store instruction writing contiguous words; the owner of a slice of
//               `cs` columns adds the partials of all workgroups in a fixed order (f64) -> its entries of
//               v = R^T s, its bits of t = sgn(v) and its share of c = sum |v| (lines 6-7).
//   hop 2       the owners publish sign bits and shares, every workgroup gathers all of them: the full t,
//               c (and ||R||_F^2 after an update), added in the same order everywhere, so that every
//               workgroup takes the same decision of line 8 without any further communication.
// Exchange: value and sequence number travel in one 8-byte relaxed agent-scope store and are read back with
// agent-scope loads; slots alternate by the parity of the sequence number.  Every wait is bounded; when one
// runs out all workgroups leave and the host reports SCD_ETIMEOUT.  No float atomics: bit-identical reruns.
#include "scd_device.h"
#include "scd_rng.h"

namespace scd {

namespace {

constexpr int kPsThreads = 512;
constexpr int kPsWaves = kPsThreads / 64;
constexpr int kPsMaxSlice = 256;   // most columns per slice of hop 1
constexpr int kPsSlot2 = 16;       // words of a hop-2 slot: up to 8 sign words, c and ||.||^2 as two halves each
constexpr int kPsMaxLast = 4;      // order 3: largest last mode (colour channels)
constexpr int kPsMaxItems2 = 6;    // hop-2 words a thread gathers: at most 256 * 12 / 512
constexpr size_t kPsMaxLds = 160 * 1024 - 512;  // dynamic LDS a launch may ask for (the compute unit has 160 KB)

template <typename TE>
struct PsVec;
template <>
struct PsVec<float> {
    typedef float4 type;
    static constexpr int N = 4;
    static constexpr int WPE = 1;  // tagged words per published value
};
template <>
struct PsVec<double> {
    typedef double2 type;
    static constexpr int N = 2;
    static constexpr int WPE = 2;
};

__device__ __forceinline__ float ps_fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
__device__ __forceinline__ double ps_fma(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float ps_flip(float x, uint32_t neg) { return __uint_as_float(__float_as_uint(x) ^ (neg << 31)); }
__device__ __forceinline__ double ps_flip(double x, uint32_t neg)
{
    return __longlong_as_double(__double_as_longlong(x) ^ ((long long)neg << 63));
}

// workgroup barrier that waits for LDS traffic only, not for the global loads of the rows in flight
__device__ __forceinline__ void ps_lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Sum over the 64 lanes, the same bits in every lane, in a fixed order and without LDS traffic: distances 1, 2,
// 4, 8 by the data-parallel lane modes (4 = mirror of half a row then reversed quads, 8 = mirror of a row then
// of half a row), 16 and 32 by the row-swap instructions of gfx950.
template <int C0, int C1>
__device__ __forceinline__ double ps_dpp_f64(double v)
{
    const long long b = __double_as_longlong(v);
    int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xFFFFFFFFll), C0, 0xF, 0xF, true);
    int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), C0, 0xF, 0xF, true);
    if constexpr (C1 != 0) {
        lo = __builtin_amdgcn_update_dpp(0, lo, C1, 0xF, 0xF, true);
        hi = __builtin_amdgcn_update_dpp(0, hi, C1, 0xF, 0xF, true);
    }
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned)lo);
}
template <int D>
__device__ __forceinline__ double ps_swap_sum_f64(double a)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(a);
    const unsigned lo = (unsigned)b, hi = (unsigned)(b >> 32);
    unsigned l0, l1, h0, h1;
    if constexpr (D == 16) {
        const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
    } else {
        const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        l0 = rl[0], l1 = rl[1], h0 = rh[0], h1 = rh[1];
    }
    return __longlong_as_double((long long)(((unsigned long long)h0 << 32) | l0)) +
           __longlong_as_double((long long)(((unsigned long long)h1 << 32) | l1));
}
// sum over groups of eight neighbouring lanes (xor butterfly over lane bits 0..2)
__device__ __forceinline__ double ps_sum8(double a)
{
    a += ps_dpp_f64<0xB1, 0>(a);      // lane ^ 1
    a += ps_dpp_f64<0x4E, 0>(a);      // lane ^ 2
    a += ps_dpp_f64<0x141, 0x1B>(a);  // lane ^ 4
    return a;
}
__device__ __forceinline__ double ps_wave_sum(double a)
{
    a += ps_dpp_f64<0xB1, 0>(a);       // lane ^ 1
    a += ps_dpp_f64<0x4E, 0>(a);       // lane ^ 2
    a += ps_dpp_f64<0x141, 0x1B>(a);   // lane ^ 4
    a += ps_dpp_f64<0x140, 0x141>(a);  // lane ^ 8
    a = ps_swap_sum_f64<16>(a);
    a = ps_swap_sum_f64<32>(a);
    return a;
}

__device__ __forceinline__ void ps_store_tagged(uint64_t* p, uint32_t v, uint32_t seq)
{
    __hip_atomic_store(p, ((uint64_t)seq << 32) | (uint64_t)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ps_load(const uint64_t* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Hop 1, one thread: the partial sums of members q, q + Q, q + 2 Q, ... < G for one column (at basep + member *
// slot1, WPE tagged words n apart), added in that order; NF members are in flight together.  false: a wait ran out.
template <int WPE, int NF>
__device__ __forceinline__ bool ps_hop1_gather(const uint64_t* basep, int q, int Q, int G, size_t slot1, int64_t n, uint32_t seq,
                                               int max_spin, double& s, int& spin)
{
#pragma nounroll
    for (int m0 = q; m0 < G; m0 += NF * Q) {
        uint64_t w[NF][WPE];
        for (;;) {
            bool fresh = true;
#pragma unroll
            for (int i = 0; i < NF; ++i) {
                const int mem = m0 + i * Q < G ? m0 + i * Q : m0;
#pragma unroll
                for (int h = 0; h < WPE; ++h) w[i][h] = ps_load(basep + (size_t)mem * slot1 + (size_t)h * n);
            }
#pragma unroll
            for (int i = 0; i < NF; ++i)
#pragma unroll
                for (int h = 0; h < WPE; ++h) fresh = fresh && ((uint32_t)(w[i][h] >> 32) == seq);
            if (fresh) break;
            if (++spin > max_spin) return false;
            __builtin_amdgcn_s_sleep(1);
        }
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            if (m0 + i * Q < G) {
                if constexpr (WPE == 1) s += (double)__uint_as_float((uint32_t)w[i][0]);
                else s += __longlong_as_double((long long)((w[i][1] << 32) | (w[i][0] & 0xFFFFFFFFull)));
            }
        }
    }
    return true;
}

// profile mode: 100 MHz ticks of workgroup 0 per phase
#define PS_TICK(slot)                                                  \
    do {                                                               \
        if (a.profile && threadIdx.x == 0) {                           \
            const uint64_t now_ = __builtin_amdgcn_s_memrealtime();    \
            sh.ticks[slot] += (int64_t)(now_ - sh.tick0);              \
            sh.tick0 = now_;                                           \
        }                                                              \
    } while (0)

struct PsShared {
    double u[2][8][kPsWaves];      // row sums of a batch [row][wave] (two parities: one barrier per batch)
    union {
        // the two exchanges use this space one after the other (barriers in between)
        struct {
            double part[kPsThreads];   // hop 1: partial sums per (member group, column)
            double v[kPsMaxSlice];     // order 3: the own slice of W_1
        };
        uint32_t scal[2 * kPsMaxLast + 2][kSpGrid];  // hop 2: low/high halves of the members' scalars
    };
    double red[2][kPsWaves];
    double redn[kPsMaxLast][kSpGrid / 64];  // order 3: wave sums of the last mode's shares
    uint32_t tw32[8];              // sign words of the own slice
    double w2part[kPsMaxLast];     // order 3: the own slice's part of the last mode's sums
    int64_t ticks[6];              // profile mode
    uint64_t tick0;
};

template <typename TE, int CPT, int RB>
struct PsTile {
    TE x[RB][CPT * PsVec<TE>::N];
    uint32_t rowsign;  // bit r: sign of row rb + r in the vector the update subtracts
};

// bits of this thread's columns from a bit array in LDS: element e of chunk c in bit c * VE + e
template <typename TE, int CPT>
__device__ __forceinline__ uint64_t ps_gather_bits(const uint64_t* bits, int64_t nch)
{
    constexpr int VE = PsVec<TE>::N;
    uint64_t out = 0;
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int64_t ch = threadIdx.x + c * kPsThreads;
        const int64_t chc = ch < nch ? ch : nch - 1;
        const int64_t col = chc * VE;  // VE divides 64: a chunk never straddles a word
        const uint64_t b = (bits[col >> 6] >> (col & 63)) & ((1ull << VE) - 1);
        out |= (ch < nch ? b : 0ull) << (c * VE);
    }
    return out;
}

__device__ __forceinline__ uint32_t ps_rowsigns(const uint8_t* sb, int rb, int nrows)
{
    uint32_t v = 0;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int i = rb + r < nrows ? rb + r : nrows - 1;
        v |= (uint32_t)(sb[i] & 1u) << r;
    }
    return v;
}

// RB rows of the block from `base` (global memory or the LDS copy), never predicated: indices past the end
// are clamped and the values dropped later.  rb: first row of the batch relative to `base`, rows: rows there.
template <typename TE, int CPT, int RB>
__device__ __forceinline__ void ps_tile_load(PsTile<TE, CPT, RB>& t, const TE* base, int64_t cols, int rb, int rows,
                                             int64_t nch, bool valid)
{
    constexpr int VE = PsVec<TE>::N;
    typedef typename PsVec<TE>::type V;
    int64_t chs[CPT];
#pragma unroll
    for (int c = 0; c < CPT; ++c) {
        const int64_t ch = threadIdx.x + c * kPsThreads;
        const int64_t chc = ch < nch ? ch : nch - 1;
        chs[c] = valid ? chc : 0;
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        int row = rb + r;
        row = row < rows ? row : rows - 1;
        row = valid ? row : 0;
        const V* rowp = (const V*)(base + (int64_t)row * cols);
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

// One batch of RB rows.  mode 0: a further alternation; 1: first subtract the finished term, write the rows
// back (to `base`: memory or the LDS copy) and sum the squares; 2: only sum the squares (start of a launch).
// full: every row of the batch and every chunk of this thread exists.  mode and full are the same for every
// thread: the branches on them are scalar.
template <typename TE, int CPT, int RB>
__device__ __forceinline__ void ps_process(PsTile<TE, CPT, RB>& t, TE* base, int64_t cols, int rb, int rows, int64_t nch,
                                           int mode, bool full, const TE* sf, uint64_t updb, TE ck, const TE* magrow, TE* acc, double& fsq,
                                           uint8_t* s_new, PsShared& sh, int parity)
{
    constexpr int VE = PsVec<TE>::N;
    constexpr int NE = CPT * VE;
    typedef typename PsVec<TE>::type V;
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    double ps[RB];
    if (!full) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const bool rok = rb + r < rows;
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const bool ok = rok && (threadIdx.x + c * kPsThreads < nch);
#pragma unroll
                for (int e = 0; e < VE; ++e) t.x[r][c * VE + e] = ok ? t.x[r][c * VE + e] : (TE)0;
            }
        }
    }
    if (mode == 1) {
        // R <- R - ck s t^T (Algorithm 5 line 10): the product of the two signs picks +ck or -ck
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const bool rok = full || (rb + r < rows);
            const uint32_t sold = (t.rowsign >> r) & 1u;
            V* rowp = (V*)(base + (int64_t)(rok ? rb + r : rows - 1) * cols);
#pragma unroll
            for (int c = 0; c < CPT; ++c) {
                const bool ok = full || (rok && (threadIdx.x + c * kPsThreads < nch));
                // real last mode (magrow != null): the magnitude depends on the column; the row of magnitudes sits in LDS
                TE mg[VE];
                if (magrow) {
                    const V mv = ((const V*)magrow)[ok ? threadIdx.x + c * kPsThreads : 0];
                    if constexpr (VE == 4) mg[0] = mv.x, mg[1] = mv.y, mg[2] = mv.z, mg[3] = mv.w;
                    else mg[0] = mv.x, mg[1] = mv.y;
                } else {
#pragma unroll
                    for (int e = 0; e < VE; ++e) mg[e] = ck;
                }
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    const TE mag = mg[e];
                    const TE d = t.x[r][c * VE + e] - ps_flip(mag, sold ^ (uint32_t)((updb >> (c * VE + e)) & 1ull));
                    t.x[r][c * VE + e] = ok ? d : (TE)0;  // padding stays zero
                }
                V v;
                if constexpr (VE == 4) v = V{t.x[r][c * 4], t.x[r][c * 4 + 1], t.x[r][c * 4 + 2], t.x[r][c * 4 + 3]};
                else v = V{t.x[r][c * 2], t.x[r][c * 2 + 1]};
                if (ok) rowp[threadIdx.x + c * kPsThreads] = v;
            }
        }
    }
    if (mode >= 1) {
        // squares in f64: large entries must not overflow, small ones must not vanish
#pragma unroll
        for (int r = 0; r < RB; ++r)
#pragma unroll
            for (int e = 0; e < NE; ++e) fsq += (double)t.x[r][e] * (double)t.x[r][e];
    }
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        TE p = 0;
#pragma unroll
        for (int e = 0; e < NE; ++e) p = ps_fma(t.x[r][e], sf[e], p);  // x * (+-1) is exact: rounds like p +- x
        ps[r] = ps_wave_sum((double)p);
    }
    if (lane == 0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) sh.u[parity][r][wv] = ps[r];
    }
    ps_lds_barrier();
    // u_r = the eight wave sums of row r added pairwise in a fixed order: lane 8 r + q reads the sum of wave q, an
    // xor butterfly over the three low lane bits leaves u_r in all eight lanes, and one ballot hands every lane
    // the signs s_i = sgn(u_i) of all rows of the batch
    const double uw = ps_sum8((lane >> 3) < RB ? sh.u[parity][(lane >> 3) & 7][lane & 7] : 0.0);
    const uint64_t negs = __ballot(uw < 0.0);
    if (lane < RB && wv == 0 && (full || rb + lane < rows)) s_new[rb + lane] = (uint8_t)((negs >> (8 * lane)) & 1ull);
#pragma unroll
    for (int r = 0; r < RB; ++r) {
        const TE sg = ((negs >> (8 * r)) & 1ull) ? (TE)-1 : (TE)1;
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[e] = ps_fma(t.x[r][e], sg, acc[e]);
    }
}

// One pass over the block: the nl rows kept in LDS, then the ng rows streamed from memory (`first` already
// holds their first batch, loaded while the previous exchange was waiting).  s_old / s_new: sign bytes of the
// block's rows before and after this pass.
template <typename TE, int CPT, int RB>
__device__ __forceinline__ void ps_pass(int mode, TE* lds_rows, int nl, TE* grows, const TE* gsafe, int ng,
                                        PsTile<TE, CPT, RB>& first,
                                        int64_t cols, uint64_t sumb, uint64_t updb, TE ck, const TE* magrow, TE* acc, double& fsq,
                                        const uint8_t* s_old, uint8_t* s_new, PsShared& sh)
{
    static_assert(RB <= 8, "ps_rowsigns packs at most 8 rows");
    constexpr int VE = PsVec<TE>::N;
    constexpr int NE = CPT * VE;
    const int64_t nch = cols / VE;
    const bool full_cols = nch == (int64_t)CPT * kPsThreads;
    int parity = 0;
    TE sf[NE];  // the signs of this thread's columns as factors +-1.0
#pragma unroll
    for (int e = 0; e < NE; ++e) sf[e] = ((sumb >> e) & 1ull) ? (TE)-1 : (TE)1;
    PsTile<TE, CPT, RB> tb;
    const int nb = (ng + RB - 1) / RB;
    (void)gsafe;
    // (the rows kept in LDS go through the second tile: it is free until the streamed rows start)
#pragma nounroll
    for (int rb = 0; rb < nl; rb += RB) {
        ps_tile_load<TE, CPT, RB>(tb, lds_rows, cols, rb, nl, nch, true);
        if (mode == 1) tb.rowsign = ps_rowsigns(s_old, rb, nl);
        ps_process<TE, CPT, RB>(tb, lds_rows, cols, rb, nl, nch, mode, full_cols && rb + RB <= nl, sf, updb, ck, magrow, acc, fsq, s_new,
                                sh, parity);
        parity ^= 1;
    }
    // two register tiles alternate, the loads of the next batch are in flight while this one is reduced; every
    // load inside the loop is unconditional
#pragma nounroll
    for (int b = 0; b < nb; b += 2) {
        const int rb = b * RB;
        ps_tile_load<TE, CPT, RB>(tb, grows, cols, rb + RB, ng, nch, b + 1 < nb);
        if (mode == 1) first.rowsign = ps_rowsigns(s_old + nl, rb, ng);
        ps_process<TE, CPT, RB>(first, grows, cols, rb, ng, nch, mode, full_cols && rb + RB <= ng, sf, updb, ck, magrow, acc, fsq,
                                s_new + nl, sh, parity);
        if (b + 1 < nb) {
            ps_tile_load<TE, CPT, RB>(first, grows, cols, rb + 2 * RB, ng, nch, b + 2 < nb);
            if (mode == 1) tb.rowsign = ps_rowsigns(s_old + nl, rb + RB, ng);
            ps_process<TE, CPT, RB>(tb, grows, cols, rb + RB, ng, nch, mode, full_cols && rb + 2 * RB <= ng, sf, updb, ck, magrow, acc,
                                    fsq, s_new + nl, sh, parity ^ 1);
        }
    }
}

// sum over the members' shares held one per thread (thread t < grid holds member t's), the same order in every
// workgroup: lanes by butterfly, then the first four waves in order.  All threads must call it.
__device__ __forceinline__ double ps_sum_members(double v, PsShared& sh, int slot)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (wv < kSpGrid / 64) {
        v = ps_wave_sum(v);
        if (lane == 0) sh.red[slot][wv] = v;
    }
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < kSpGrid / 64; ++q) t += sh.red[slot][q];
    return t;
}

// The same for the cnt <= kPsMaxLast shares of the last mode of an order-3 tensor at once (one barrier for all;
// each sum in the order ps_sum_members takes).  All threads must call it.
__device__ __forceinline__ void ps_sum_members_n(const double (&v)[kPsMaxLast], int cnt, PsShared& sh, double (&out)[kPsMaxLast])
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    if (wv < kSpGrid / 64) {
#pragma unroll
        for (int c = 0; c < kPsMaxLast; ++c) {
            const double t = ps_wave_sum(c < cnt ? v[c] : 0.0);
            if (lane == 0) sh.redn[c][wv] = t;
        }
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < kPsMaxLast; ++c) {
        double t = 0.0;
#pragma unroll
        for (int q = 0; q < kSpGrid / 64; ++q) t += sh.redn[c][q];
        out[c] = t;
    }
}

// Column signs of the level-0 view of an order-3 tensor: bit q = s2[q / n3] xor s3[q % n3] (Algorithm 12 lines
// 5-7: the sign of the tensor product of the other modes' vectors).  A thread forms 32 consecutive bits from the
// at most 33 rows of s2 that they touch (n2 bits of s2 are valid, the rest of its last word is zero).
__device__ __forceinline__ void ps_kron_bits(uint64_t* out, int64_t n, int n3, const uint64_t* s2, int n2, uint64_t s3)
{
    uint32_t* o32 = (uint32_t*)out;
    const int w2 = (n2 + 63) / 64;
    const int nh = (int)((n + 63) / 64) * 2;  // half words of the array
    const float rn3 = 1.0f / (float)n3;
    for (int h = threadIdx.x; h < nh; h += kPsThreads) {
        const int q0 = h * 32;
        // q0 / n3 by a float product, exact here: (q0 + 0.5) / n3 is at least 0.5 / n3 away from an integer and
        // q0 stays below 2^20 + 64
        const int j = (int)(((float)q0 + 0.5f) * rn3);
        int cc = q0 - j * n3, jj = 0;
        const int wi = j >> 6, sh = j & 63;
        const uint64_t lo = s2[wi < w2 ? wi : w2 - 1], hi = s2[wi + 1 < w2 ? wi + 1 : w2 - 1];
        const uint64_t x = sh ? (lo >> sh) | (hi << (64 - sh)) : lo;  // rows j, j + 1, ... from bit 0
        uint32_t o = 0;
#pragma unroll 8
        for (int b = 0; b < 32; ++b) {
            o |= (((uint32_t)(x >> jj) ^ (uint32_t)(s3 >> cc)) & 1u) << b;
            if (++cc == n3) {
                cc = 0;
                ++jj;
            }
        }
        const int64_t valid = n - q0;  // bits of this half word inside the array: the padding stays zero
        o32[h] = valid >= 32 ? o : (valid > 0 ? o & ((1u << (int)valid) - 1u) : 0u);
    }
}

// SC: real last mode (a template parameter: the all-signs kernels then carry none of its code).
template <typename TE, int CPT, int RB, bool SC>
__global__ void __launch_bounds__(kPsThreads) pstream_kernel(PStreamArgs a)
{
    constexpr int VE = PsVec<TE>::N;
    constexpr int NE = CPT * VE;
    constexpr int WPE = PsVec<TE>::WPE;
    typedef typename PsVec<TE>::type V;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int g = blockIdx.x, G = a.grid;
    const int64_t n = a.n, nch = n / VE;
    const int r0 = g * a.rpw;
    const int nrows = (int)((int64_t)r0 + a.rpw <= a.m ? a.rpw : a.m - r0);  // >= 1 for every workgroup of the grid
    const int nl = nrows < a.lds_rows ? nrows : a.lds_rows;                 // rows kept in LDS
    const int ng = nrows - nl;                                              // rows streamed every alternation
    const int nw = a.nw;
    const bool tensor = a.n3 > 0;               // order 3: the columns are (mode 1) x (mode 2), n = n2 * n3
    const int n3 = a.n3, w2 = a.w2;             // w2: words of a mode-1 sign vector (n2 bits)

    extern __shared__ __align__(16) unsigned char ps_lds[];
    // layout: [rows kept in LDS][one row of partial sums][column signs t][t_0 of the coming term][sign bytes x 2]
    //         [order 3: s^(2) and its random start][fixed part]
    TE* lds_rows = (TE*)ps_lds;
    size_t off = (((size_t)a.lds_rows * (size_t)n * sizeof(TE)) + 15) & ~(size_t)15;
    TE* pub = (TE*)(ps_lds + off);
    off += (((size_t)n * sizeof(TE)) + 15) & ~(size_t)15;
    uint64_t* t_cur = (uint64_t*)(ps_lds + off);
    off += (size_t)nw * 8;
    uint64_t* t_rng = (uint64_t*)(ps_lds + off);
    off += (size_t)nw * 8;
    uint64_t* s2_cur = (uint64_t*)(ps_lds + off);
    off += (size_t)w2 * 8;
    uint8_t* sbuf0 = ps_lds + off;
    off += ((size_t)a.rpw + 15) & ~(size_t)15;
    uint8_t* sbuf1 = ps_lds + off;
    off += ((size_t)a.rpw + 15) & ~(size_t)15;
    PsShared& sh = *(PsShared*)(ps_lds + off);

    TE* const grows = (TE*)a.R + ((int64_t)r0 + nl) * n;  // first streamed row (only dereferenced when ng > 0)
    TE* const gfirst = ng > 0 ? grows : (TE*)a.R + (int64_t)r0 * n;

    // ---- the block's first rows into LDS (read from memory once per launch)
    {
        const V* src = (const V*)((const TE*)a.R + (int64_t)r0 * n);
        V* dst = (V*)lds_rows;
        const int64_t tot = (int64_t)nl * nch;
        for (int64_t i = tid; i < tot; i += kPsThreads) dst[i] = src[i];
    }
    // the random start of the first term (Algorithm 4 line 2; Algorithm 12 line 1 for the modes after the first)
    uint64_t s3_cur = 0;  // order 3: the signs of the last mode (at most 64), the same in every thread
    if (tensor) {
        for (int p = tid; p < w2; p += kPsThreads) s2_cur[p] = rng_word_masked(a.seed, (uint64_t)a.k_start, 1u, p, a.n2);
        s3_cur = rng_word_masked(a.seed, (uint64_t)a.k_start, 2u, 0, n3);
        __syncthreads();
        ps_kron_bits(t_rng, n, n3, s2_cur, a.n2, s3_cur);
    } else {
        for (int p = tid; p < nw; p += kPsThreads) t_rng[p] = rng_word_masked(a.seed, (uint64_t)a.k_start, 1u, p, n);
    }
    for (int p = tid; p < nw; p += kPsThreads) t_cur[p] = 0;
    for (int i = tid; i < a.rpw; i += kPsThreads) sbuf0[i] = sbuf1[i] = 0;
    __syncthreads();

    // columns this workgroup reduces in hop 1: [c0, c0 + ncol)
    const int cs = a.cs;
    const int64_t c0 = (int64_t)g * cs;
    const int ncol = (int)(c0 >= n ? 0 : (n - c0 < cs ? n - c0 : cs));
    const int Q = kPsThreads / cs;                // member groups of the hop-1 reduction (cs <= 256)
    const int unit = tensor ? n3 : 1;             // columns per sign bit that a slice publishes
    const int sbits = cs / unit;                  // sign bits of a slice (a multiple of 8)
    const int tw = (sbits + 31) / 32;             // sign words of a slice
    const int sbytes = sbits >> 3;
    const int nsc = tensor ? 2 * n3 : 2;          // words of scalars per slot: c (or the n3 mode sums) as halves
    const size_t slot1 = (size_t)n * WPE;         // words of a hop-1 slot

    int64_t k = a.k_start;
    int64_t alternations = 0, updates = 0, spins = 0;
    uint32_t seq = a.seq;
    int j = 0, warn = 0, sp = 0, mode = 2;  // 2: start pass (squares only), 0: alternation, 1: update
    bool final_pass = k >= a.w_target;
    double c_prev = -INFINITY;
    TE ck = (TE)0;
    const double total = (double)a.m * (double)a.n;
    uint64_t bcur = 0, brng = ps_gather_bits<TE, CPT>(t_rng, nch);

    PsTile<TE, CPT, RB> first;
    ps_tile_load<TE, CPT, RB>(first, gfirst, n, 0, ng > 0 ? ng : 1, nch, ng > 0);
    if (tid == 0) {
        for (int i = 0; i < 6; ++i) sh.ticks[i] = 0;
        sh.tick0 = __builtin_amdgcn_s_memrealtime();
    }

    for (;;) {
        // ================= the pass over the block
        TE acc[NE];
#pragma unroll
        for (int e = 0; e < NE; ++e) acc[e] = 0;
        double fsq = 0.0;
        uint8_t* s_old = sp ? sbuf1 : sbuf0;
        uint8_t* s_new = sp ? sbuf0 : sbuf1;
        ps_pass<TE, CPT, RB>(mode, lds_rows, nl, grows, gfirst, ng, first, n, mode == 0 ? bcur : brng, bcur, ck, SC ? pub : (TE*)nullptr, acc, fsq,
                             s_old, s_new, sh);
        sp ^= 1;  // s_new is the current s
        PS_TICK(0);
        ++alternations;
        ++seq;
        const bool with_norm = mode != 0;

        // ================= hop 1: publish the partial column sums, reduce the own slice
        // (through LDS, so that every store instruction writes 512 consecutive tagged words: the 16-byte chunks
        // of a thread are 2 KB apart, and partial-line stores to the fabric are what costs)
#pragma unroll
        for (int c = 0; c < CPT; ++c) {
            const int64_t ch = tid + c * kPsThreads;
            if (ch < nch) {
                V v;
                if constexpr (VE == 4) v = V{acc[c * 4], acc[c * 4 + 1], acc[c * 4 + 2], acc[c * 4 + 3]};
                else v = V{acc[c * 2], acc[c * 2 + 1]};
                ((V*)pub)[ch] = v;
            }
        }
        if (with_norm) {
            fsq = ps_wave_sum(fsq);
            if (lane == 0) sh.red[1][wv] = fsq;
        }
        __syncthreads();
        {
            uint64_t* mine = a.xp + ((size_t)(seq & 1u) * G + g) * slot1;
#pragma nounroll
            for (int64_t col = tid; col < n; col += kPsThreads) {
                if constexpr (WPE == 1) {
                    ps_store_tagged(mine + col, __float_as_uint((float)pub[col]), seq);
                } else {
                    const uint64_t b = (uint64_t)__double_as_longlong((double)pub[col]);
                    ps_store_tagged(mine + col, (uint32_t)b, seq);
                    ps_store_tagged(mine + n + col, (uint32_t)(b >> 32), seq);
                }
            }
        }
        // the first streamed batch of the next pass does not depend on the exchange: its loads fly meanwhile
        ps_tile_load<TE, CPT, RB>(first, gfirst, n, 0, ng > 0 ? ng : 1, nch, ng > 0);
        PS_TICK(1);
        for (int d = 0; d < a.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
        bool ok = true;
        double vj = 0.0;
        {
            const int q = tid / cs, jc = tid - q * cs;
            double s = 0.0;
            if (q < Q && jc < ncol) {
                const uint64_t* basep = a.xp + ((size_t)(seq & 1u) * G) * slot1 + (size_t)(c0 + jc);
                int spin = 0;
                // members q, q + Q, ... in that order; 16 in flight when a thread has more than 8 of them (one-word
                // values only: 32 words in flight would not fit the registers)
                if (WPE == 1 && G > 8 * Q) ok = ps_hop1_gather<WPE, WPE == 1 ? 16 : 8>(basep, q, Q, G, slot1, n, seq, a.max_spin, s, spin);
                else ok = ps_hop1_gather<WPE, 8>(basep, q, Q, G, slot1, n, seq, a.max_spin, s, spin);
                spins += spin;
            }
            sh.part[tid] = s;
            if (tid < 8) sh.tw32[tid] = 0;
        }
        if (__syncthreads_or(ok ? 0 : 1)) {
            if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
            return;
        }
        PS_TICK(2);
        // v at the own columns: L neighbouring lanes share a column, each adds every L-th member group in order,
        // a butterfly joins them
        {
            const int L = cs <= 64 ? 8 : (cs <= 128 ? 4 : 2);
            const int jc = tid / L, ql = tid - jc * L;
            double pq[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int q = ql + i * L;
                pq[i] = (jc < ncol && q < Q) ? sh.part[q * cs + jc] : 0.0;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) vj += pq[i];
            vj += ps_dpp_f64<0xB1, 0>(vj);                    // lane ^ 1
            if (L >= 4) vj += ps_dpp_f64<0x4E, 0>(vj);        // lane ^ 2
            if (L >= 8) vj += ps_dpp_f64<0x141, 0x1B>(vj);    // lane ^ 4
            const bool mine = jc < ncol && ql == 0;
            if (!tensor) {
                // t_l = sgn(v_l), share of c = sum |v_l| (Algorithm 4 lines 6-7)
                if (mine && vj < 0.0) atomicOr(&sh.tw32[jc >> 5], 1u << (jc & 31));
                const double ca = ps_wave_sum(mine ? fabs(vj) : 0.0);
                if (lane == 0) sh.red[0][wv] = ca;
            } else if (mine) {
                sh.v[jc] = vj;  // the slice of W_1 = a x_1 s^(1): whole rows of the n2 x n3 array
            }
        }
        __syncthreads();
        if (tensor) {
            // mode 2 on the own rows of W_1: s^(2)_j = sgn(sum_c W_1[j][c] s^(3)_c) with the last mode's signs of the
            // previous sweep (Algorithm 12: modes before the current one new, modes after it old), then this
            // slice's part of the last mode's sums W_2[c] = sum_j s^(2)_j W_1[j][c]
            const int nr2 = ncol / n3;
            if (tid < nr2) {
                double u2 = 0.0;
                for (int c = 0; c < n3; ++c) u2 += ((s3_cur >> c) & 1ull) ? -sh.v[tid * n3 + c] : sh.v[tid * n3 + c];
                if (u2 < 0.0) atomicOr(&sh.tw32[tid >> 5], 1u << (tid & 31));
            }
            __syncthreads();
            if (tid < n3) {
                double w2c = 0.0;
                for (int j0 = 0; j0 < nr2; j0 += 8) {
                    double x[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) x[i] = sh.v[(j0 + i < nr2 ? j0 + i : nr2 - 1) * n3 + tid];
                    const uint32_t bits = sh.tw32[j0 >> 5] >> (j0 & 31);  // (eight rows never straddle a word)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (j0 + i < nr2) w2c += ((bits >> i) & 1u) ? -x[i] : x[i];
                }
                sh.w2part[tid] = w2c;
            }
            __syncthreads();
        }
        PS_TICK(3);
        // ================= hop 2: publish the slice's sign bits and scalars, gather everybody's
        {
            uint64_t* mine = a.xq + ((size_t)(seq & 1u) * G + g) * kPsSlot2;
            if (tid < tw) ps_store_tagged(mine + tid, sh.tw32[tid], seq);
            if (!tensor) {
                if (tid == 64) {
                    double cq[kPsWaves], cshare = 0.0;
#pragma unroll
                    for (int q = 0; q < kPsWaves; ++q) cq[q] = sh.red[0][q];
#pragma unroll
                    for (int q = 0; q < kPsWaves; ++q) cshare += cq[q];
                    const uint64_t b = (uint64_t)__double_as_longlong(cshare);
                    ps_store_tagged(mine + tw, (uint32_t)b, seq);
                    ps_store_tagged(mine + tw + 1, (uint32_t)(b >> 32), seq);
                }
            } else if (tid >= 64 && tid < 64 + n3) {
                const uint64_t b = (uint64_t)__double_as_longlong(sh.w2part[tid - 64]);
                ps_store_tagged(mine + tw + 2 * (tid - 64), (uint32_t)b, seq);
                ps_store_tagged(mine + tw + 2 * (tid - 64) + 1, (uint32_t)(b >> 32), seq);
            }
            if (with_norm && tid == 128) {
                double f = 0.0;
#pragma unroll
                for (int q = 0; q < kPsWaves; ++q) f += sh.red[1][q];
                const uint64_t b = (uint64_t)__double_as_longlong(f);
                ps_store_tagged(mine + tw + nsc, (uint32_t)b, seq);
                ps_store_tagged(mine + tw + nsc + 1, (uint32_t)(b >> 32), seq);
            }
        }
        for (int d = 0; d < a.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
        {
            const int per = tw + nsc + (with_norm ? 2 : 0);
            const int items = G * per;
            int where[kPsMaxItems2];  // member * kPsSlot2 + word, or -1
#pragma unroll
            for (int it = 0; it < kPsMaxItems2; ++it) {
                const int idx = tid + it * kPsThreads;
                const int mem = idx / per, wd = idx - mem * per;
                where[it] = idx < items ? mem * kPsSlot2 + wd : -1;
            }
            const uint64_t* xb = a.xq + (size_t)(seq & 1u) * G * kPsSlot2;
            uint64_t w[kPsMaxItems2];
#pragma unroll
            for (int it = 0; it < kPsMaxItems2; ++it) w[it] = (uint64_t)(where[it] >= 0 ? ~seq : seq) << 32;
            int spin = 0;
            for (;;) {
                bool fresh = true;
#pragma unroll
                for (int it = 0; it < kPsMaxItems2; ++it)
                    if ((uint32_t)(w[it] >> 32) != seq) w[it] = ps_load(xb + where[it]);
#pragma unroll
                for (int it = 0; it < kPsMaxItems2; ++it) fresh = fresh && ((uint32_t)(w[it] >> 32) == seq);
                if (fresh) break;
                if (++spin > a.max_spin) {
                    ok = false;
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            spins += spin;
            if (ok) {
                // sign bits: the columns' t (matrix) or the rows' s^(2) (order 3), member after member
                uint8_t* tbytes = tensor ? (uint8_t*)s2_cur : (uint8_t*)t_cur;
                const int nbytes = tensor ? w2 * 8 : nw * 8;
#pragma unroll
                for (int it = 0; it < kPsMaxItems2; ++it) {
                    if (where[it] >= 0) {
                        const int mem = where[it] / kPsSlot2, wd = where[it] % kPsSlot2;
                        const uint32_t v = (uint32_t)w[it];
                        if (wd < tw) {
                            const int b0 = mem * sbytes + 4 * wd;
#pragma unroll
                            for (int b = 0; b < 4; ++b)
                                if (4 * wd + b < sbytes && b0 + b < nbytes) tbytes[b0 + b] = (uint8_t)(v >> (8 * b));
                        } else {
                            sh.scal[wd - tw][mem] = v;
                        }
                    }
                }
            }
        }
        if (__syncthreads_or(ok ? 0 : 1)) {
            if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
            return;
        }
        PS_TICK(4);
        // the scalars: sums of the members' shares, the same order in every workgroup
        double c_tot = 0.0, f_tot = 0.0;
        double wl[kPsMaxLast] = {0.0, 0.0, 0.0, 0.0};  // order 3: the last mode's sums W_2[c] of this sweep
        auto share = [&](int slot) {
            return tid < G ? __longlong_as_double((long long)(((uint64_t)sh.scal[2 * slot + 1][tid] << 32) | sh.scal[2 * slot][tid]))
                           : 0.0;
        };
        if (!tensor) {
            c_tot = ps_sum_members(share(0), sh, 0);
        } else {
            // last mode: s^(3)_c = sgn(W_2[c]); the cut value is <s, a> = sum_c |W_2[c]| (Algorithm 12 line 10)
            uint64_t s3n = 0;
            double sv[kPsMaxLast];
#pragma unroll
            for (int c = 0; c < kPsMaxLast; ++c) sv[c] = c < n3 ? share(c) : 0.0;
            ps_sum_members_n(sv, n3, sh, wl);
#pragma unroll
            for (int c = 0; c < kPsMaxLast; ++c) {
                if (c < n3) {
                    if (wl[c] < 0.0) s3n |= 1ull << c;
                    c_tot += fabs(wl[c]);
                }
            }
            s3_cur = s3n;
            ps_kron_bits(t_cur, n, n3, s2_cur, a.n2, s3_cur);
        }
        if (with_norm) f_tot = ps_sum_members(share(nsc / 2), sh, 1);
        if (with_norm && g == 0 && tid == 0) a.trace[k] = sqrt(f_tot);
        if (final_pass) break;
        ++j;
        __syncthreads();  // (order 3: t_cur was just rebuilt)
        bcur = ps_gather_bits<TE, CPT>(t_cur, nch);  // this thread's bits of t_j: row sums of the next pass, or the update
        const bool conv = (c_tot <= c_prev) || (j >= a.max_iters);  // Algorithm 4 line 8 / Algorithm 12 line 11
        if (conv) {
            // the term is complete: append it (Algorithm 5 lines 7-9); the next pass subtracts it (line 10)
            if (!(c_tot <= c_prev)) warn = 1;
            const double ckd = c_tot / total;
            ck = (TE)ckd;
            if constexpr (SC) {
                // real last mode: the coefficient of slice c is <s (x) t, r[..., c]> / (n_1 n_2) = W_2[c] / (n_1 n_2), the
                // least squares coefficient for these sign vectors; its sign is s^(3)_c, so the update of the next
                // pass subtracts its magnitude with the signs of the all-signs term.  Stored rounded; what is stored
                // is what is subtracted.  The magnitudes go, column by column, into the LDS row that holds the partial
                // sums during an exchange (it is free during a pass).
                TE coef[kPsMaxLast];
#pragma unroll
                for (int c = 0; c < kPsMaxLast; ++c) coef[c] = (TE)(wl[c] / (total / (double)n3));
                const float rn3 = 1.0f / (float)n3;
                for (int64_t col = tid; col < n; col += kPsThreads) {
                    const int cc = (int)col - (int)(((float)col + 0.5f) * rn3) * n3;  // col mod n3 (exact below 2^20)
                    TE v = coef[0];
#pragma unroll
                    for (int c = 1; c < kPsMaxLast; ++c) v = cc == c ? coef[c] : v;
                    pub[col] = v < (TE)0 ? -v : v;
                }
                if (g == 0 && tid < n3) {
                    TE v = coef[0];
#pragma unroll
                    for (int c = 1; c < kPsMaxLast; ++c) v = tid == c ? coef[c] : v;
                    ((TE*)a.c)[k * n3 + tid] = v;
                }
            }
            {
                // own rows' bits of the first mode: the rows of a workgroup need not start at a word boundary
                const uint8_t* sc = sp ? sbuf1 : sbuf0;
                unsigned long long* Sk = (unsigned long long*)(a.S + k * a.mw);
                for (int i0 = wv * 64; i0 < nrows; i0 += kPsThreads) {
                    const int i = i0 + lane;
                    const uint64_t word = __ballot(i < nrows && sc[i < nrows ? i : 0] != 0);
                    if (lane == 0 && word) {
                        const int64_t bit0 = (int64_t)r0 + i0;
                        const int shft = (int)(bit0 & 63);
                        atomicOr(Sk + (bit0 >> 6), (unsigned long long)(word << shft));
                        if (shft && (word >> (64 - shft))) atomicOr(Sk + (bit0 >> 6) + 1, (unsigned long long)(word >> (64 - shft)));
                    }
                }
            }
            if (g == 0) {
                if (!tensor) {
                    for (int p = tid; p < nw; p += kPsThreads) a.T[k * nw + p] = t_cur[p];
                } else {
                    for (int p = tid; p < w2; p += kPsThreads) a.T[k * w2 + p] = s2_cur[p];
                    if (tid == 0 && !SC) a.S3[k] = s3_cur;
                }
                if (tid == 0) {
                    if (!SC) ((TE*)a.c)[k] = ck;
                    a.iters[k] = j;
                }
            }
            ++k;
            ++updates;
            j = 0;
            c_prev = -INFINITY;
            mode = 1;
            final_pass = k >= a.w_target;
            __syncthreads();  // t_cur / s2_cur were read above
            // the random start of the coming term
            if (tensor) {
                for (int p = tid; p < w2; p += kPsThreads) s2_cur[p] = rng_word_masked(a.seed, (uint64_t)k, 1u, p, a.n2);
                s3_cur = rng_word_masked(a.seed, (uint64_t)k, 2u, 0, n3);
                __syncthreads();
                ps_kron_bits(t_rng, n, n3, s2_cur, a.n2, s3_cur);
            } else {
                for (int p = tid; p < nw; p += kPsThreads) t_rng[p] = rng_word_masked(a.seed, (uint64_t)k, 1u, p, n);
            }
            __syncthreads();
            brng = ps_gather_bits<TE, CPT>(t_rng, nch);
        } else {
            c_prev = c_tot;
            mode = 0;
        }
        // what this iteration read from LDS is next written after the barriers of the coming pass and hops
        __syncthreads();
        PS_TICK(5);
    }

    // ---- the rows kept in LDS go back to memory
    __syncthreads();
    {
        V* dst = (V*)((TE*)a.R + (int64_t)r0 * n);
        const V* src = (const V*)lds_rows;
        const int64_t tot = (int64_t)nl * nch;
        for (int64_t i = tid; i < tot; i += kPsThreads) dst[i] = src[i];
    }
    if (g == 0 && tid == 0) {
        a.res->k = k;
        a.res->alternations = alternations;
        a.res->updates = updates;
        a.res->seq_u = seq;
        a.res->warn = warn;
        a.res->spins = spins;
        for (int i = 0; i < 6; ++i) a.res->ticks[i] = sh.ticks[i];
    }
}

template <typename TE, int CPT, int RB, bool SC>
hipError_t ps_launch_k(const PStreamArgs& a, size_t lds_bytes, hipStream_t st)
{
    auto kern = pstream_kernel<TE, CPT, RB, SC>;
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
    if (e != hipSuccess) return e;
    // every workgroup of the grid must be resident at once: one per compute unit is enough
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kPsThreads, lds_bytes);
    if (e != hipSuccess) return e;
    if ((int64_t)per_cu * prop.multiProcessorCount < a.grid) return hipErrorCooperativeLaunchTooLarge;
    hipLaunchKernelGGL(kern, dim3(a.grid), dim3(kPsThreads), lds_bytes, st, a);
    return hipGetLastError();
}

template <typename TE, int CPT>
hipError_t ps_launch_rb(const PStreamArgs& a, size_t lds_bytes, hipStream_t st)
{
    constexpr int VE = PsVec<TE>::N;
    // rows per register tile: at most 32 registers per tile (two tiles are live; more rows per batch would
    // mean fewer joins across the waves, but with 48 registers per tile the register allocator spills 64-bit
    // values to odd register pairs, which this compiler then rejects)
    constexpr int kRegsPerRow = CPT * VE * (int)sizeof(TE) / 4;
    constexpr int RB = kRegsPerRow > 16 ? 1 : (kRegsPerRow > 8 ? 2 : (kRegsPerRow > 4 ? 4 : 8));
    if (a.scalars && a.n3 > 0) return ps_launch_k<TE, CPT, RB, true>(a, lds_bytes, st);
    return ps_launch_k<TE, CPT, RB, false>(a, lds_bytes, st);
}

template <typename TE>
hipError_t ps_launch(const PStreamArgs& a, size_t lds_bytes, hipStream_t st)
{
    constexpr int VE = PsVec<TE>::N;
    const int64_t nch = a.n / VE;
    const int cpt = (int)((nch + kPsThreads - 1) / kPsThreads);
    switch (cpt) {
        case 1: return ps_launch_rb<TE, 1>(a, lds_bytes, st);
        case 2: return ps_launch_rb<TE, 2>(a, lds_bytes, st);
        case 3:
        case 4: return ps_launch_rb<TE, 4>(a, lds_bytes, st);
        case 5:
        case 6: return ps_launch_rb<TE, 6>(a, lds_bytes, st);
        case 7:
        case 8: return ps_launch_rb<TE, 8>(a, lds_bytes, st);
        default: return hipErrorInvalidValue;
    }
}

// chunks per thread the kernel is instantiated with for rows of nch chunks (0: too long)
int ps_cpt(int64_t nch)
{
    const int64_t cpt = (nch + kPsThreads - 1) / kPsThreads;
    if (cpt <= 2) return (int)cpt;
    if (cpt <= 8) return (int)((cpt + 1) / 2 * 2);
    return 0;
}

size_t ps_fixed_lds(int64_t n, size_t es, int64_t n2, int rpw)
{
    const size_t nw = (size_t)((n + 63) / 64), w2 = (size_t)((n2 + 63) / 64);
    return (((size_t)n * es + 15) & ~(size_t)15) + 2 * nw * 8 + w2 * 8 + 2 * (((size_t)rpw + 15) & ~(size_t)15) +
           sizeof(PsShared) + 64;
}

}  // namespace

// Geometry of a launch on `limit` workgroups, or false when the engine does not take the shape.  Matrices, and
// order-3 tensors with a last mode of at most 4 (seen as n_1 x (n_2 n_3)), whose rows are a multiple of 16 bytes
// and at most 64 KB long, on enough workgroups for slices of at most 256 columns.
bool pstream_supported(scd_dtype dt, int order, const int64_t* dims, int limit, PStreamGeometry* geo)
{
    if ((order != 2 && order != 3) || limit < 1) return false;
    const int64_t m = dims[0], n = order == 2 ? dims[1] : dims[1] * dims[2];
    const int64_t n3 = order == 3 ? dims[2] : 0, n2 = order == 3 ? dims[1] : 0;
    if (order == 3 && (n3 < 1 || n3 > kPsMaxLast || n2 < 1)) return false;
    const int ve = dt == SCD_F32 ? 4 : 2;
    const size_t es = dt == SCD_F32 ? 4 : 8;
    if (m < 1 || n < ve || (n % ve) || m > (1ll << 30) || n > (1 << 20)) return false;
    if (ps_cpt(n / ve) == 0) return false;
    if (limit > kSpGrid) limit = kSpGrid;
    const int64_t rpw = (m + limit - 1) / limit;
    const int64_t grid = (m + rpw - 1) / rpw;
    const int64_t unit = order == 3 ? 8 * n3 : 8;  // slices hold whole bytes of sign bits (of whole rows of W_1)
    int64_t cs = (n + grid - 1) / grid;
    cs = (cs + unit - 1) / unit * unit;
    if (cs > kPsMaxSlice || rpw > (1 << 20)) return false;
    const size_t fixed = ps_fixed_lds(n, es, n2, (int)rpw);
    if (fixed > kPsMaxLds) return false;
    int64_t lds_rows = (int64_t)((kPsMaxLds - fixed) / ((size_t)n * es));
    if (lds_rows > rpw) lds_rows = rpw;
    if (geo) {
        geo->grid = (int)grid;
        geo->rpw = (int)rpw;
        geo->cs = (int)cs;
        geo->lds_rows = (int)lds_rows;
        geo->lds_bytes = ((((size_t)lds_rows * (size_t)n * es) + 15) & ~(size_t)15) + fixed;
        geo->xp_bytes = (size_t)2 * (size_t)grid * (size_t)n * (dt == SCD_F32 ? 1 : 2) * 8;
        geo->xq_bytes = (size_t)2 * (size_t)grid * kPsSlot2 * 8;
    }
    return true;
}

hipError_t launch_pstream(const PStreamArgs& a, scd_dtype dt, size_t lds_bytes, hipStream_t st)
{
    return dt == SCD_F32 ? ps_launch<float>(a, lds_bytes, st) : ps_launch<double>(a, lds_bytes, st);
}

}  // namespace scd
