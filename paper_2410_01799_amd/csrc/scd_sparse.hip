// Cached, sparsified alternation (Section 3.1 of arXiv 2410.01799) as one persistent launch.
//
// After the first alternation of a term only a few signs change per alternation, so
//     R t_j     = R t_{j-1}     + 2 * sum over flipped columns l of t_j[l] * R[:, l]
//     R^T s_j   = R^T s_{j-1}   + 2 * sum over flipped rows    i of s_j[i] * R[i, :]
// and an alternation touches a few per cent of the matrix instead of all of it.  The paper keeps the
// matrix and its transpose so that both kinds of slices are contiguous; so does this engine (R and RT
// in HBM, both updated when a term is subtracted).
//
// G workgroups (up to 256, one per compute unit: the whole device by default, a share
// of it when several decompositions run side by side).  Workgroup g owns the slice I_g of the rows
// (its entries of u = R t) and the slice J_g of the columns (its entries of v = R^T s), in f64.
//   term start   dense: rows I_g of R   -> subtract the finished term (Algorithm 5 line 10), ||R||^2,
//                        u = R t_0; all-gather of s;   rows J_g of RT -> subtract, v = R^T s; all-gather of t
//   afterwards   sparse: u[I_g] += 2 sum_f +-RT[l_f][I_g]; all-gather of s;
//                        v[J_g] += 2 sum_f +-R[i_f][J_g];  all-gather of t and of the shares of c
// The all-gather is the tagged exchange of the register-resident engine (one 8-byte relaxed
// agent-scope store per word: 32 payload bits + 32-bit sequence number; readers poll with loads that
// bypass the non-coherent caches; slots alternate by sequence parity; every wait is bounded).
// Flipped indices are compacted in ascending order and added in a fixed order: results are
// bit-identical from run to run.
// A second kernel (further down) delays the subtraction of finished terms as Section 3.2 does: pending
// terms live in LDS, the products are corrected from their bitsets, one pass flushes the list and, while
// it is at it, forms the first products R' t_0 of the next terms (their random starts are known in advance).
#include "scd_device.h"
#include "scd_rng.h"

namespace scd {

namespace {

constexpr int kSpThreads = 512;
constexpr int kSpWaves = kSpThreads / kWave;
constexpr int kSpPayload = 16;                    // payload words per slot (32 sign bits each)
constexpr int kSpSlotUsed = kSpPayload + 2;       // + one double as two tagged halves
// Every workgroup reads every slot: slots 4 KB apart land on different memory channels, so that the
// 256 x 256 reads of one exchange do not queue up at a handful of them.
constexpr int kSpSlot = 512;
constexpr int kSpListCap = 32 * kSpThreads;       // flips handled per compaction round: one 32-bit word per thread
constexpr size_t kSpMaxLds = 150 * 1024;          // most dynamic LDS a launch may ask for
// Words a thread may have to gather: grid * (ceil(slice / 32) + 2) over the supported pairs, where
// grid * slice <= 65536 + 8 * grid: at most 67584 / 32 + 256 + 512 = 2880 words for the 512 threads
// (sparse_supported checks it).
constexpr int kSpMaxItems = 6;

// The value of lane (l ^ D) for D = 1, 2, 4, 8 by the data-parallel lane modes (vector-unit latency; a
// ds_bpermute would cost an LDS round trip per step of a dependent chain).
template <int D>
__device__ __forceinline__ double sp_lane_xor_f64(double v)
{
    const long long b = __double_as_longlong(v);
    int lo = (int)(b & 0xFFFFFFFFll), hi = (int)(b >> 32);
    if constexpr (D == 1) {  // quad_perm 1,0,3,2
        lo = __builtin_amdgcn_update_dpp(0, lo, 0xB1, 0xF, 0xF, true);
        hi = __builtin_amdgcn_update_dpp(0, hi, 0xB1, 0xF, 0xF, true);
    } else if constexpr (D == 2) {  // quad_perm 2,3,0,1
        lo = __builtin_amdgcn_update_dpp(0, lo, 0x4E, 0xF, 0xF, true);
        hi = __builtin_amdgcn_update_dpp(0, hi, 0x4E, 0xF, 0xF, true);
    } else if constexpr (D == 4) {  // mirror of half a row (l ^ 7), then quad_perm 3,2,1,0 (l ^ 3)
        lo = __builtin_amdgcn_update_dpp(0, __builtin_amdgcn_update_dpp(0, lo, 0x141, 0xF, 0xF, true), 0x1B, 0xF, 0xF, true);
        hi = __builtin_amdgcn_update_dpp(0, __builtin_amdgcn_update_dpp(0, hi, 0x141, 0xF, 0xF, true), 0x1B, 0xF, 0xF, true);
    } else {  // D == 8: mirror of a row (l ^ 15), then of half a row (l ^ 7)
        static_assert(D == 8, "distance within a row of 16 lanes");
        lo = __builtin_amdgcn_update_dpp(0, __builtin_amdgcn_update_dpp(0, lo, 0x140, 0xF, 0xF, true), 0x141, 0xF, 0xF, true);
        hi = __builtin_amdgcn_update_dpp(0, __builtin_amdgcn_update_dpp(0, hi, 0x140, 0xF, 0xF, true), 0x141, 0xF, 0xF, true);
    }
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned)lo);
}

// Sum over the 64 lanes, the same bits in every lane: distances 1, 2, 4, 8 by the lane modes above, 16 and 32
// by the row-swap instructions of gfx950 (swapping the odd rows of one copy with the even rows of another
// leaves the two partners of every lane in the two results, in the same order for both partners).
__device__ __forceinline__ double sp_wave_sum(double a)
{
    a += sp_lane_xor_f64<1>(a);
    a += sp_lane_xor_f64<2>(a);
    a += sp_lane_xor_f64<4>(a);
    a += sp_lane_xor_f64<8>(a);
    {
        const unsigned long long b = (unsigned long long)__double_as_longlong(a);
        const unsigned lo = (unsigned)b, hi = (unsigned)(b >> 32);
        const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
        a = __longlong_as_double((long long)(((unsigned long long)rh[0] << 32) | rl[0])) +
            __longlong_as_double((long long)(((unsigned long long)rh[1] << 32) | rl[1]));
    }
    {
        const unsigned long long b = (unsigned long long)__double_as_longlong(a);
        const unsigned lo = (unsigned)b, hi = (unsigned)(b >> 32);
        const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
        const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
        a = __longlong_as_double((long long)(((unsigned long long)rh[0] << 32) | rl[0])) +
            __longlong_as_double((long long)(((unsigned long long)rh[1] << 32) | rl[1]));
    }
    return a;
}

// a[l] + a[l ^ 16] and a[l] + a[l ^ 32], the same bits in both partners (see sp_wave_sum)
__device__ __forceinline__ double sp_sum_xor16(double a)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(a);
    const unsigned lo = (unsigned)b, hi = (unsigned)(b >> 32);
    const auto rl = __builtin_amdgcn_permlane16_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane16_swap(hi, hi, false, false);
    return __longlong_as_double((long long)(((unsigned long long)rh[0] << 32) | rl[0])) +
           __longlong_as_double((long long)(((unsigned long long)rh[1] << 32) | rl[1]));
}
__device__ __forceinline__ double sp_sum_xor32(double a)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(a);
    const unsigned lo = (unsigned)b, hi = (unsigned)(b >> 32);
    const auto rl = __builtin_amdgcn_permlane32_swap(lo, lo, false, false);
    const auto rh = __builtin_amdgcn_permlane32_swap(hi, hi, false, false);
    return __longlong_as_double((long long)(((unsigned long long)rh[0] << 32) | rl[0])) +
           __longlong_as_double((long long)(((unsigned long long)rh[1] << 32) | rl[1]));
}

// Sum of an int over the 64 lanes (every lane gets it) and inclusive prefix sum across the lanes, both
// without LDS traffic.  The scan is the classic one of this architecture: shifts by 1, 2, 4, 8 within each
// row of 16 lanes (lanes without a source add zero), then lane 15 of rows 0 and 2 is added to rows 1 and 3,
// then lane 31 to rows 2 and 3.
__device__ __forceinline__ int sp_wave_sum_int(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);                                                    // l ^ 1
    v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);                                                    // l ^ 2
    v += __builtin_amdgcn_update_dpp(0, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true), 0x1B, 0xF, 0xF, true);   // l ^ 4
    v += __builtin_amdgcn_update_dpp(0, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true), 0x141, 0xF, 0xF, true);  // l ^ 8
    {
        const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        v = (int)(r[0] + r[1]);
    }
    {
        const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        v = (int)(r[0] + r[1]);
    }
    return v;
}
__device__ __forceinline__ int sp_wave_scan_int(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

__device__ __forceinline__ uint32_t sp_bits4(const uint32_t* bits, int64_t col)
{
    // the bits of `col .. col+3` (col is a multiple of 4, so they sit in one word)
    return (bits[col >> 5] >> (col & 31)) & 0xFu;
}

template <typename TE>
struct SpVec;
template <>
struct SpVec<float> {
    typedef float4 type;
    static constexpr int N = 4;
};
template <>
struct SpVec<double> {
    typedef double2 type;
    static constexpr int N = 2;
};

__device__ __forceinline__ float sp_flip(float x, uint32_t neg) { return __uint_as_float(__float_as_uint(x) ^ (neg << 31)); }
__device__ __forceinline__ double sp_flip(double x, uint32_t neg)
{
    return __longlong_as_double(__double_as_longlong(x) ^ ((long long)neg << 63));
}

// Shared-memory carve-up of one workgroup.
struct SpShared {
    uint32_t* sA;      // sign bits of the rows, two buffers (current / other)
    uint32_t* sB;
    uint32_t* tA;      // sign bits of the columns
    uint32_t* tB;
    uint16_t* list;    // compacted flips of one round: index within the round | new sign << 15
    double* accu;      // u on I_g
    double* accv;      // v on J_g
    double* red;       // [kSpThreads] partial sums of the sparse accumulation / per-wave scratch
    uint32_t* scal;    // [2][kSpGrid][2] gathered scalars (lo, hi halves)
    int* scan;         // [kSpWaves + 1]
};

// Dense pass over `nrows` consecutive rows of Y (row length ld, a multiple of 16 bytes): optionally
// subtract ck * rowsign * colsign, sum the squares, and form the signed row sums with `sumbits`.
template <typename TE>
__device__ void sp_dense_rows(TE* __restrict__ Y, int64_t ld, int64_t row0, int nrows, bool upd,
                              const uint32_t* rowbits_upd, const uint32_t* colbits_upd, TE ck,
                              const uint32_t* colbits_sum, double* acc, double& fsq_out, double* red)
{
    constexpr int VE = SpVec<TE>::N;
    constexpr int RB = 8;
    typedef typename SpVec<TE>::type V;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int64_t nch = ld / VE;
    double fsq = 0.0;
    for (int rb = 0; rb < nrows; rb += RB) {
        double ps[RB];
        uint32_t sr[RB];
        V* rowp[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int rr = rb + r < nrows ? rb + r : nrows - 1;
            const int64_t row = row0 + rr;
            ps[r] = 0.0;
            sr[r] = upd ? ((rowbits_upd[row >> 5] >> (row & 31)) & 1u) : 0u;
            rowp[r] = (V*)(Y + row * ld);
        }
        for (int64_t c = tid; c < nch; c += kSpThreads) {
            const int64_t col = c * VE;
            const uint32_t bsum = sp_bits4(colbits_sum, col & ~3ll) >> (col & 3);
            const uint32_t bupd = upd ? (sp_bits4(colbits_upd, col & ~3ll) >> (col & 3)) : 0u;
            V v[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) v[r] = rowp[r][c];
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                if (rb + r >= nrows) continue;
                TE x[VE];
                if constexpr (VE == 4) {
                    x[0] = v[r].x; x[1] = v[r].y; x[2] = v[r].z; x[3] = v[r].w;
                } else {
                    x[0] = v[r].x; x[1] = v[r].y;
                }
                if (upd) {
#pragma unroll
                    for (int e = 0; e < VE; ++e) x[e] = x[e] - sp_flip(ck, sr[r] ^ ((bupd >> e) & 1u));
                    V o;
                    if constexpr (VE == 4) o = V{x[0], x[1], x[2], x[3]};
                    else o = V{x[0], x[1]};
                    rowp[r][c] = o;
#pragma unroll
                    for (int e = 0; e < VE; ++e) fsq += (double)x[e] * (double)x[e];
                }
#pragma unroll
                for (int e = 0; e < VE; ++e) ps[r] += (double)sp_flip(x[e], (bsum >> e) & 1u);
            }
        }
#pragma unroll
        for (int r = 0; r < RB; ++r) ps[r] = sp_wave_sum(ps[r]);
        __syncthreads();  // `red` may still be read from the previous batch
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < RB; ++r) red[wv * RB + r] = ps[r];
        }
        __syncthreads();
        if (tid < RB && rb + tid < nrows) {
            double s = 0.0;
            for (int q = 0; q < kSpWaves; ++q) s += red[q * RB + tid];
            acc[rb + tid] = s;
        }
    }
    // squares: per-wave sums, then in wave order
    fsq = sp_wave_sum(fsq);
    __syncthreads();
    if (lane == 0) red[wv] = fsq;
    __syncthreads();
    double f = 0.0;
    for (int q = 0; q < kSpWaves; ++q) f += red[q];
    fsq_out = f;
    __syncthreads();
}

// part + the signed entries of flips f, f + Q, .., f + (Z - 1) Q of the list (those below total), added in
// that order; every load is issued before the first add
template <typename TE, int Z>
__device__ __forceinline__ double sp_gather_batch(const TE* __restrict__ ycol, int64_t ld, int64_t ibase, const uint16_t* list,
                                                  int f, int Q, int total, double part)
{
    uint16_t en[Z];
    TE val[Z];
#pragma unroll
    for (int z = 0; z < Z; ++z) en[z] = f + z * Q < total ? list[f + z * Q] : (uint16_t)0;
#pragma unroll
    for (int z = 0; z < Z; ++z) val[z] = ycol[(ibase + (en[z] & 0x3FFF)) * ld];
#pragma unroll
    for (int z = 0; z < Z; ++z) part += f + z * Q < total ? (double)sp_flip(val[z], (uint32_t)(en[z] >> 15)) : 0.0;
    return part;
}

// acc[e] += 2 * sum over the indices i whose sign changed (cur xor prev) of sign_cur(i) * Y[i][off + e],
// e < len.  Flipped indices are compacted in ascending order, one 32-bit word of sign bits per thread
// and round, and every thread adds its share of the list in order.
template <typename TE>
__device__ void sp_accumulate_flips(const TE* __restrict__ Y, int64_t ld, int64_t off, int len, const uint32_t* cur,
                                    const uint32_t* prev, int64_t nbits, double* acc, SpShared& sh, int64_t& nflips)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    int slp = 16;
    while (slp < len) slp <<= 1;  // lanes per flip: power of two >= len (len <= kSpThreads)
    const int Q = kSpThreads / slp;
    const int e = tid & (slp - 1), q = tid / slp;
    const bool active = e < len;
    const TE* ycol = Y + off + e;
    double part = 0.0;
    const int64_t nwords = (nbits + 31) >> 5;
    for (int64_t w0 = 0; w0 < nwords; w0 += kSpThreads) {
        // ---- compaction of this round's flips
        const int64_t wi = w0 + tid;
        const uint32_t cw = wi < nwords ? cur[wi] : 0u;
        const uint32_t x = wi < nwords ? (cw ^ prev[wi]) : 0u;
        const int cnt = __popc(x);
        const int incl = sp_wave_scan_int(cnt);
        // the list and the scan cells of the previous round are free (before the first round they have been
        // since the barriers that closed the previous call)
        if (w0 > 0) __syncthreads();
        if (lane == kWave - 1) sh.scan[wv + 1] = incl;
        __syncthreads();
        // (all eight cells are loaded before any is added: a loop with a run-time bound would pay an LDS
        // latency per turn)
        int sc[kSpWaves];
#pragma unroll
        for (int i = 0; i < kSpWaves; ++i) sc[i] = sh.scan[i + 1];
        int base = 0, total = 0;
#pragma unroll
        for (int i = 0; i < kSpWaves; ++i) {
            total += sc[i];
            base += i < wv ? sc[i] : 0;
        }
        int pos = base + incl - cnt;
        uint32_t bits = x;
        while (bits) {
            const int b = __ffs(bits) - 1;
            bits &= bits - 1;
            sh.list[pos++] = (uint16_t)((tid * 32 + b) | (((cw >> b) & 1u) << 15));
        }
        __syncthreads();
        nflips += total;
        // ---- gather: thread (e, q) takes flips q, q+Q, ... in order.  All loads of a batch are issued before
        // the first is used, and the batch is sized to what is left (16, 8, 4 or 2 per thread), so a round
        // of up to 16 Q flips costs one trip to memory; slots past the end re-read a valid row and add zero.
        if (active) {
            const int64_t ibase = w0 * 32;
            int f0 = 0;
            while (f0 < total) {
                const int left = (total - f0 + Q - 1) / Q;  // loads the busiest thread still has to make
                if (left > 8) {
                    part = sp_gather_batch<TE, 16>(ycol, ld, ibase, sh.list, f0 + q, Q, total, part);
                    f0 += 16 * Q;
                } else if (left > 4) {
                    part = sp_gather_batch<TE, 8>(ycol, ld, ibase, sh.list, f0 + q, Q, total, part);
                    f0 += 8 * Q;
                } else if (left > 2) {
                    part = sp_gather_batch<TE, 4>(ycol, ld, ibase, sh.list, f0 + q, Q, total, part);
                    f0 += 4 * Q;
                } else {
                    part = sp_gather_batch<TE, 2>(ycol, ld, ibase, sh.list, f0 + q, Q, total, part);
                    f0 += 2 * Q;
                }
            }
        }
    }
    // the lanes of a wave that hold the same entry are joined first (their groups in ascending order of the
    // distance), then the waves in order
    if (slp <= 16) part = sp_sum_xor16(part);
    if (slp <= 32) part = sp_sum_xor32(part);
    __syncthreads();
    if (slp >= kWave) sh.red[tid] = part;
    else if (lane < slp) sh.red[wv * slp + e] = part;
    __syncthreads();
    if (tid < len) {
        const int groups = slp >= kWave ? Q : kSpWaves;  // 8 or fewer
        double gsum[kSpWaves];
#pragma unroll
        for (int z = 0; z < kSpWaves; ++z) gsum[z] = z < groups ? sh.red[z * slp + tid] : 0.0;  // loaded together
        double s = 0.0;
#pragma unroll
        for (int z = 0; z < kSpWaves; ++z) s += gsum[z];
        acc[tid] += 2.0 * s;
    }
    // No barrier here: a thread reads back only its own entry of acc, and every path from here passes a barrier
    // before sh.red is written again (the pending-term products, the exchange, the sum of |v| all start or end
    // with one).
}

__device__ __forceinline__ void sp_store_tagged(uint64_t* p, uint32_t v, uint32_t seq)
{
    __hip_atomic_store(p, ((uint64_t)seq << 32) | (uint64_t)v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Publish this workgroup's slice of sign bits (taken from acc < 0) and, if asked, one scalar, then read every
// workgroup's: the full bit vector lands in `dest`, the scalars in sh.scal.  Returns false on time-out.
// `fence`: this exchange also hands over ordinary data (the rows of R or RT this workgroup has just
// rewritten): the writes are released to the whole device before anything is published, and the
// caches are invalidated after the gather, because the L2 of one XCD does not see another's writes.
__device__ bool sp_exchange(const SparseArgs& a, uint32_t seq, const double* acc, int len, int slice, int64_t total_bits,
                            double sc0, bool has_scalar, uint32_t* dest, SpShared& sh, int& spins, bool fence)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int g = blockIdx.x;
    if (fence) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __syncthreads();
    }
    uint64_t* mine = a.xbuf + ((size_t)(seq & 1u) * kSpGrid + g) * kSpSlot;
    const int words = (slice + 31) >> 5;  // payload words every workgroup publishes
    // ---- publish: one ballot per 64 slice entries
    for (int b = wv * kWave; b < slice; b += kSpThreads) {
        const int e = b + lane;
        const uint64_t bal = __ballot(e < len && acc[e] < 0.0);
        if (lane == 0) {
            sp_store_tagged(mine + (b >> 5), (uint32_t)bal, seq);
            if (b + 32 < slice) sp_store_tagged(mine + (b >> 5) + 1, (uint32_t)(bal >> 32), seq);
        }
    }
    if (has_scalar && tid == kSpThreads - 1) {
        const uint64_t b0 = (uint64_t)__double_as_longlong(sc0);
        sp_store_tagged(mine + kSpPayload + 0, (uint32_t)b0, seq);
        sp_store_tagged(mine + kSpPayload + 1, (uint32_t)(b0 >> 32), seq);
    }
    for (int d = 0; d < a.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
    // ---- gather: the payload words (+ the two halves of the scalar) of each of the a.grid members, spread
    // over the threads.  Every workgroup polls every slot and every word read or written is a trip through
    // the fabric, so a word that is not needed is not sent: an exchange without a scalar took 5.9 us with the
    // two unused scalars of an earlier layout in it and takes 2.9 us without (14336 x 4096, 256 workgroups).
    const int per = words + (has_scalar ? 2 : 0);
    const int items = a.grid * per;
    uint64_t w[kSpMaxItems];
    // where this thread's words lie (member * kSpSlot + word; -1: none), worked out once.  item / per by a
    // float product: (item + 0.5) / per is at least 0.5 / 18 away from an integer, items stay below 4608.
    int where[kSpMaxItems];
    {
        const float rper = 1.0f / (float)per;
#pragma unroll
        for (int it = 0; it < kSpMaxItems; ++it) {
            const int idx = tid + it * kSpThreads;
            const int mem = (int)(((float)idx + 0.5f) * rper), k = idx - mem * per;
            const int word = k < words ? k : kSpPayload + (k - words);
            where[it] = idx < items ? mem * kSpSlot + word : -1;
        }
    }
    const uint64_t* xb = a.xbuf + (size_t)(seq & 1u) * kSpGrid * kSpSlot;
    bool ok = true;
    int spin = 0;
#pragma unroll
    for (int it = 0; it < kSpMaxItems; ++it) w[it] = (uint64_t)(where[it] >= 0 ? ~seq : seq) << 32;  // missing: not the current tag
    for (;;) {
        bool fresh = true;
        // only the words that have not arrived yet are read again
#pragma unroll
        for (int it = 0; it < kSpMaxItems; ++it) {
            if ((uint32_t)(w[it] >> 32) != seq)
                w[it] = __hip_atomic_load(xb + where[it], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
        for (int it = 0; it < kSpMaxItems; ++it) fresh = fresh && ((uint32_t)(w[it] >> 32) == seq);
        if (fresh) break;
        if (++spin > a.max_spin) {
            ok = false;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    spins += spin;
    if (fence) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    if (ok) {
        uint8_t* dbytes = (uint8_t*)dest;
        const int sbytes = slice >> 3;                      // bytes of one member's slice (slice is a multiple of 8)
        const int64_t tbytes = (total_bits + 7) >> 3;
#pragma unroll
        for (int it = 0; it < kSpMaxItems; ++it) {
            if (where[it] >= 0) {
                const int mem = where[it] / kSpSlot, word = where[it] % kSpSlot;  // (kSpSlot is a power of two)
                const uint32_t v = (uint32_t)w[it];
                if (word < kSpPayload) {
                    const int64_t b0 = (int64_t)mem * sbytes + 4 * word;
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        if (4 * word + b < sbytes && b0 + b < tbytes) dbytes[b0 + b] = (uint8_t)(v >> (8 * b));
                } else {
                    sh.scal[mem * 2 + (word - kSpPayload)] = v;  // low, high half of the scalar
                }
            }
        }
    }
    return !__syncthreads_or(ok ? 0 : 1);
}

// Sum of one gathered scalar over the members, in a fixed order; every thread gets the same bits.
__device__ double sp_sum_scalar(const SpShared& sh, double* scratch, int grid)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    if (tid < kWave) {
        double s = 0.0;
        for (int g = lane; g < grid; g += kWave) {
            const uint32_t lo = sh.scal[g * 2], hi = sh.scal[g * 2 + 1];
            s += __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
        }
        s = sp_wave_sum(s);
        if (lane == 0) scratch[0] = s;
    }
    __syncthreads();
    const double r = scratch[0];
    __syncthreads();
    return r;
}

template <typename TE>
__global__ void __launch_bounds__(kSpThreads) sparse_kernel(SparseArgs a)
{
    extern __shared__ __align__(16) unsigned char sp_lds[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int g = blockIdx.x;
    const int64_t m = a.m, n = a.n;
    const int64_t mwords32 = (m + 31) >> 5, nwords32 = (n + 31) >> 5;

    SpShared sh;
    {
        size_t o = 0;
        auto take = [&](size_t bytes) {
            unsigned char* p = sp_lds + o;
            o += (bytes + 15) & ~(size_t)15;
            return p;
        };
        sh.sA = (uint32_t*)take((size_t)mwords32 * 4 + 8);
        sh.sB = (uint32_t*)take((size_t)mwords32 * 4 + 8);
        sh.tA = (uint32_t*)take((size_t)nwords32 * 4 + 8);
        sh.tB = (uint32_t*)take((size_t)nwords32 * 4 + 8);
        sh.list = (uint16_t*)take((size_t)kSpListCap * 2);
        sh.accu = (double*)take((size_t)kSpThreads * 8);
        sh.accv = (double*)take((size_t)kSpThreads * 8);
        sh.red = (double*)take((size_t)kSpThreads * 8);
        sh.scal = (uint32_t*)take((size_t)2 * kSpGrid * 2 * 4);
        sh.scan = (int*)take((size_t)(kSpWaves + 1) * 4);
    }
    for (int64_t i = tid; i < mwords32 + 2; i += kSpThreads) {
        sh.sA[i] = 0;
        sh.sB[i] = 0;
    }
    for (int64_t i = tid; i < nwords32 + 2; i += kSpThreads) {
        sh.tA[i] = 0;
        sh.tB[i] = 0;
    }
    __syncthreads();
    uint32_t *s_cur = sh.sA, *s_oth = sh.sB, *t_cur = sh.tA, *t_oth = sh.tB;

    const int rs = a.rs, cs = a.cs;
    const int64_t i0 = (int64_t)g * rs < m ? (int64_t)g * rs : m;
    const int rlen = (int)((i0 + rs < m ? i0 + rs : m) - i0);
    const int64_t j0 = (int64_t)g * cs < n ? (int64_t)g * cs : n;
    const int clen = (int)((j0 + cs < n ? j0 + cs : n) - j0);
    TE* R = (TE*)a.R;
    TE* RT = (TE*)a.RT;
    const double total = (double)m * (double)n;

    int64_t k = a.k_start;
    uint32_t seq = a.seq;
    int alternations = 0, updates = 0, warn = 0, spins = 0;
    int64_t flips = 0, flips_rows = 0;
    bool pending = false;  // a finished term waits to be subtracted
    double ck = 0.0;
    const bool prof = a.profile && g == 0 && tid == 0;
    int64_t tick[6] = {0, 0, 0, 0, 0, 0};
    uint64_t tk = prof ? wall_clock64() : 0;
#define SP_TICK(i)                              \
    if (prof) {                                 \
        const uint64_t now = wall_clock64();    \
        tick[i] += (int64_t)(now - tk);         \
        tk = now;                               \
    }

    for (;;) {
        if (k >= a.w_target && !pending) break;
        // ================= start of term k (dense): subtract the finished term, first alternation
        // t_0 from the keyed stream (Algorithm 4 line 2), into the other column buffer
        for (int64_t i = tid; i < nwords32; i += kSpThreads) {
            uint32_t v = (uint32_t)(rng_word(a.seed, (uint64_t)k, 1u, (uint64_t)(i >> 1)) >> (32 * (i & 1)));
            const int64_t rem = n - i * 32;
            if (rem < 32) v &= (1u << rem) - 1u;
            t_oth[i] = v;
        }
        __syncthreads();
        const TE ckt = (TE)ck;
        double fsq = 0.0, dummy = 0.0;
        // rows I_g of R: R <- R - ck s t^T (Algorithm 5 line 10), squares, u = R t_0 (Algorithm 4 line 5)
        if (rlen > 0) sp_dense_rows<TE>(R, n, i0, rlen, pending, s_cur, t_cur, ckt, t_oth, sh.accu, fsq, sh.red);
        const bool was_pending = pending;
        if (!sp_exchange(a, ++seq, sh.accu, rlen, rs, m, fsq, true, s_oth, sh, spins, was_pending)) {
            if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
            return;
        }
        ++alternations;
        if (pending) {
            const double F = sp_sum_scalar(sh, sh.red, a.grid);
            if (g == 0 && tid == 0) a.trace[k] = sqrt(F);
        }
        // rows J_g of RT (columns of R): same update, v = R^T s_1 (Algorithm 4 line 6)
        const bool last = k >= a.w_target;
        if (clen > 0 && (pending || !last))
            sp_dense_rows<TE>(RT, m, j0, clen, pending, t_cur, s_cur, ckt, s_oth, sh.accv, dummy, sh.red);
        if (pending) ++updates;
        pending = false;
        SP_TICK(0)
        if (last) break;
        // the old term's signs are dead: s_cur <- s_1, t_cur <- t_0
        {
            uint32_t* z = s_cur; s_cur = s_oth; s_oth = z;
            z = t_cur; t_cur = t_oth; t_oth = z;
        }
        int j = 0;
        double c_prev = -INFINITY;
        bool handover = was_pending;  // RT was rewritten: the next exchange carries the fences
        for (;;) {
            // ---- finish the column half: t = sgn(v), c = sum |v| (Algorithm 4 lines 6-7), all-gather
            double cabs = (tid < clen) ? fabs(sh.accv[tid]) : 0.0;
            cabs = sp_wave_sum(cabs);
            __syncthreads();
            if (lane == 0) sh.red[wv] = cabs;
            __syncthreads();
            double cpart = 0.0;
            for (int q = 0; q < kSpWaves; ++q) cpart += sh.red[q];
            __syncthreads();
            if (!sp_exchange(a, ++seq, sh.accv, clen, cs, n, cpart, true, t_oth, sh, spins, handover)) {
                if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
                return;
            }
            handover = false;
            {
                uint32_t* z = t_cur; t_cur = t_oth; t_oth = z;  // t_cur = t_j, t_oth = t_{j-1}
            }
            ++j;
            SP_TICK(1)
            const double c = sp_sum_scalar(sh, sh.red, a.grid);
            // ---- Algorithm 4 line 8
            if (c <= c_prev || j >= a.max_iters) {
                if (!(c <= c_prev)) warn = 1;
                ck = c / total;
                if (g == 0) {
                    for (int p = tid; p < a.mw; p += kSpThreads)
                        a.S[k * a.mw + p] = (uint64_t)s_cur[2 * p] | ((uint64_t)(2 * p + 1 < mwords32 ? s_cur[2 * p + 1] : 0u) << 32);
                    if (tid == 0) {
                        ((TE*)a.c)[k] = (TE)ck;
                        a.iters[k] = j;
                    }
                }
                if (g == (a.grid > 1 ? 1 : 0)) {
                    for (int p = tid; p < a.nw; p += kSpThreads)
                        a.T[k * a.nw + p] = (uint64_t)t_cur[2 * p] | ((uint64_t)(2 * p + 1 < nwords32 ? t_cur[2 * p + 1] : 0u) << 32);
                }
                pending = true;
                ++k;
                break;
            }
            c_prev = c;
            // ---- row half, sparse: u += 2 sum over flipped columns (rows of RT), s = sgn(u), all-gather
            SP_TICK(2)
            sp_accumulate_flips<TE>(RT, m, i0, rlen, t_cur, t_oth, n, sh.accu, sh, flips);
            SP_TICK(3)
            if (!sp_exchange(a, ++seq, sh.accu, rlen, rs, m, 0.0, false, s_oth, sh, spins, false)) {
                if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
                return;
            }
            SP_TICK(4)
            {
                uint32_t* z = s_cur; s_cur = s_oth; s_oth = z;  // s_cur = s_{j+1}
            }
            ++alternations;
            // ---- column half, sparse: v += 2 sum over flipped rows (rows of R)
            sp_accumulate_flips<TE>(R, n, j0, clen, s_cur, s_oth, m, sh.accv, sh, flips_rows);
            SP_TICK(5)
        }
    }
    if (g == 0 && tid == 0) {
        a.res->k = k;
        a.res->alternations = alternations;
        a.res->updates = updates;
        a.res->seq_u = seq;
        a.res->seq_v = seq;
        a.res->warn = warn;
        a.res->spins = spins;
        a.res->flips = flips;
        a.res->flips_rows = flips_rows;
        for (int i = 0; i < 6; ++i) a.res->ticks[i] = tick[i];
    }
}

// =================================================================================================
// Delayed updates (Section 3.2): the finished terms are not subtracted at once.  The two copies hold
// R' = R_k + sum over the pending terms of c_j s_j t_j^T; every product with the true remainder is the
// product with R' minus a correction from the pending terms' bitsets,
//     (R_k t)_i   = (R' t)_i   - sum_j c_j s_j[i] <t_j, t>,      <t_j, t> = n - 2 popcount(t_j xor t),
//     (R_k^T s)_l = (R'^T s)_l - sum_j c_j t_j[l] <s_j, s>,
// and when the list is full (or the launch ends) all pending terms are subtracted in one pass over each
// copy, term after term per entry, so the copies end up bit-identical to those of immediate updates.
// The dense start of a term then only reads.  ||R_k||_F between flushes follows from the cut value:
// ||R - c s t^T||^2 = ||R||^2 - 2 c <s, R t> + c^2 mn; at a flush it is measured again.

struct SpPending {
    uint32_t* PS;        // [width][ps_stride] row sign bits of the pending terms
    uint32_t* PT;        // [width][pt_stride] column sign bits
    double* coef;        // [32] coefficients as stored (rounded to the element type)
    double* ej;          // [32] coefficient times inner product, per half step
    double* effu;        // [kSpThreads] u of the true remainder on this workgroup's rows
    double* effv;        // [kSpThreads] v on its columns
    uint32_t* rowmask;   // [4]
    uint32_t* T0;        // [kSpAhead][pt_stride] random starts t_0 of the next terms
    double* U0;          // [kSpAhead][kSpThreads] their first products R' t_0 on this workgroup's rows
    int ps_stride, pt_stride;
};

// Between two flushes the stored copy R' does not change, so the first product R' t_0 of each of the next
// terms (t_0 is a keyed random vector, known in advance) can be formed in the pass that flushes: that pass
// reads R anyway, and the dense start of those terms then reads only the transposed copy.
constexpr int kSpAhead = 8;

// ej[j] = coef[j] * <p_j, cur> for the np pending vectors of one side, 0 for j >= np
__device__ void sp_pending_dots(const uint32_t* P, int stride, int nwords32, int64_t nbits, const uint32_t* cur, int np,
                                int width, const double* coef, double* ej)
{
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    for (int j = wv; j < ((width + 7) & ~7); j += kSpWaves) {
        if (j >= np) {
            if (lane == 0) ej[j] = 0.0;
            continue;
        }
        int cnt = 0;
        for (int p = lane; p < nwords32; p += kWave) cnt += __popc(P[j * stride + p] ^ cur[p]);
        cnt = sp_wave_sum_int(cnt);
        if (lane == 0) ej[j] = coef[j] * (double)(nbits - 2 * (int64_t)cnt);
    }
    __syncthreads();
}

// eff[tid] = acc[tid] - sum_j ej[j] * (sign of pending vector j at this thread's entry), in the order
// j = 0..31 (ej is zero past the last pending term); `own` holds those signs, bit j for term j.
// Every thread reads back only its own entry, so no barrier follows.
__device__ __forceinline__ void sp_effective(const double* acc, int len, uint32_t own, const double* ej, int width,
                                             double* eff)
{
    const int tid = threadIdx.x;
    if (tid < len) {
        double v = acc[tid];
        for (int j0 = 0; j0 < width; j0 += 8) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const double e = ej[j0 + j];
                v -= ((own >> (j0 + j)) & 1u) ? -e : e;
            }
        }
        eff[tid] = v;
    }
}

// Flush: rows row0 .. row0+nrows-1 of Y (row length ld) lose the np pending terms (possibly none), one after
// the other per entry (sign of term j at (row, col) = Prow_j[row] xor Pcol_j[col]); the squares of what is
// left are summed, and the signed row sums with each of the nvec <= NV bit vectors sums + j * sstride are
// formed: out[j * kSpThreads + row].  Columns are taken in tiles of one 16-byte chunk per thread, so that a
// thread keeps its columns' pending signs in registers while it streams down the rows.
template <typename TE, int NV>
__device__ void sp_flush_rows(TE* __restrict__ Y, int64_t ld, int64_t row0, int nrows, const uint32_t* Prow, int prs,
                              const uint32_t* Pcol, int pcs, int np, const double* coef, const uint32_t* sums, int sstride,
                              int nvec, double* out, double& fsq_out, double* red, uint32_t* rowmask)
{
    constexpr int VE = SpVec<TE>::N;
    constexpr int RB = 4;
    typedef typename SpVec<TE>::type V;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int64_t nch = ld / VE;
    double fsq = 0.0;
    if (tid < nrows)
        for (int j = 0; j < nvec; ++j) out[j * kSpThreads + tid] = 0.0;
    for (int64_t c0 = 0; c0 < nch; c0 += kSpThreads) {
        const int64_t c = c0 + tid;
        const bool active = c < nch;
        const int64_t col = (active ? c : 0) * VE;
        uint32_t cm[VE];
#pragma unroll
        for (int e = 0; e < VE; ++e) cm[e] = 0u;
        for (int j = 0; j < np; ++j) {
            const uint32_t bits = Pcol[j * pcs + (int)(col >> 5)] >> (col & 31);
#pragma unroll
            for (int e = 0; e < VE; ++e) cm[e] |= ((bits >> e) & 1u) << j;
        }
        uint32_t bsum = 0u;  // four bits per sum vector: its signs at this thread's columns
#pragma unroll
        for (int j = 0; j < NV; ++j)
            if (j < nvec) bsum |= ((sp_bits4(sums + j * sstride, col & ~3ll) >> (col & 3)) & 0xFu) << (4 * j);
        for (int rb = 0; rb < nrows; rb += RB) {
            __syncthreads();  // rowmask and red are free again
            if (tid < RB) {
                const int rr = rb + tid < nrows ? rb + tid : nrows - 1;
                const int64_t row = row0 + rr;
                uint32_t mk = 0u;
                for (int j = 0; j < np; ++j) mk |= ((Prow[j * prs + (int)(row >> 5)] >> (row & 31)) & 1u) << j;
                rowmask[tid] = mk;
            }
            __syncthreads();
            double ps[RB][NV];
            V v[RB];
            V* rowp[RB];
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                const int rr = rb + r < nrows ? rb + r : nrows - 1;
                rowp[r] = (V*)(Y + (row0 + rr) * ld);
#pragma unroll
                for (int j = 0; j < NV; ++j) ps[r][j] = 0.0;
                v[r] = rowp[r][active ? c : 0];
            }
#pragma unroll
            for (int r = 0; r < RB; ++r) {
                if (rb + r >= nrows || !active) continue;
                TE x[VE];
                if constexpr (VE == 4) {
                    x[0] = v[r].x; x[1] = v[r].y; x[2] = v[r].z; x[3] = v[r].w;
                } else {
                    x[0] = v[r].x; x[1] = v[r].y;
                }
                if (np > 0) {
                    uint32_t z[VE];
#pragma unroll
                    for (int e = 0; e < VE; ++e) z[e] = rowmask[r] ^ cm[e];
                    for (int j = 0; j < np; ++j) {
                        const TE ck = (TE)coef[j];
#pragma unroll
                        for (int e = 0; e < VE; ++e) x[e] = x[e] - sp_flip(ck, (z[e] >> j) & 1u);
                    }
                    V o;
                    if constexpr (VE == 4) o = V{x[0], x[1], x[2], x[3]};
                    else o = V{x[0], x[1]};
                    rowp[r][c] = o;
                }
                double xd[VE];
#pragma unroll
                for (int e = 0; e < VE; ++e) {
                    xd[e] = (double)x[e];
                    fsq += xd[e] * xd[e];
                }
#pragma unroll
                for (int j = 0; j < NV; ++j) {
                    if (j >= nvec) continue;
#pragma unroll
                    for (int e = 0; e < VE; ++e) ps[r][j] += sp_flip(xd[e], (bsum >> (4 * j + e)) & 1u);
                }
            }
            if constexpr (RB * NV == 32) {
                // 32 sums over the wave at once: at distance 32, 16, .., 2 a lane hands half of what it holds to
                // its partner and keeps the other half (31 exchanges instead of 32 x 6); after the last
                // distance the pair of lanes 2 i, 2 i + 1 holds the sum number i
                double vv[32];
#pragma unroll
                for (int r = 0; r < RB; ++r)
#pragma unroll
                    for (int j = 0; j < NV; ++j) vv[r * NV + j] = ps[r][j];
#pragma unroll
                for (int h = 16; h >= 1; h >>= 1) {
                    const bool upper = (lane & (2 * h)) != 0;  // distance 2 h: 32, 16, 8, 4, 2
#pragma unroll
                    for (int i = 0; i < h; ++i) {
                        const double send = upper ? vv[i] : vv[i + h];
                        const double keep = upper ? vv[i + h] : vv[i];
                        vv[i] = keep + __shfl_xor(send, 2 * h, kWave);
                    }
                }
                vv[0] += __shfl_xor(vv[0], 1, kWave);
                if ((lane & 1) == 0) red[wv * 32 + (lane >> 1)] = vv[0];
            } else {
#pragma unroll
                for (int r = 0; r < RB; ++r)
#pragma unroll
                    for (int j = 0; j < NV; ++j) {
                        if (j >= nvec) continue;
                        const double t = sp_wave_sum(ps[r][j]);
                        if (lane == 0) red[(wv * RB + r) * NV + j] = t;
                    }
            }
            __syncthreads();
            if (tid < RB * NV) {
                const int r = tid / NV, j = tid % NV;
                if (rb + r < nrows && j < nvec) {
                    double t = 0.0;
                    for (int q = 0; q < kSpWaves; ++q) t += red[(q * RB + r) * NV + j];
                    out[j * kSpThreads + rb + r] += t;
                }
            }
        }
    }
    fsq = sp_wave_sum(fsq);
    __syncthreads();
    if (lane == 0) red[wv] = fsq;
    __syncthreads();
    double f = 0.0;
    for (int q = 0; q < kSpWaves; ++q) f += red[q];
    fsq_out = f;
    __syncthreads();
}

template <typename TE>
__global__ void __launch_bounds__(kSpThreads) sparse_delay_kernel(SparseArgs a)
{
    extern __shared__ __align__(16) unsigned char sp_lds[];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int g = blockIdx.x;
    const int64_t m = a.m, n = a.n;
    const int64_t mwords32 = (m + 31) >> 5, nwords32 = (n + 31) >> 5;
    const int width = a.delay_width;

    SpShared sh;
    SpPending pd;
    {
        size_t o = 0;
        auto take = [&](size_t bytes) {
            unsigned char* p = sp_lds + o;
            o += (bytes + 15) & ~(size_t)15;
            return p;
        };
        sh.sA = (uint32_t*)take((size_t)mwords32 * 4 + 8);
        sh.sB = (uint32_t*)take((size_t)mwords32 * 4 + 8);
        sh.tA = (uint32_t*)take((size_t)nwords32 * 4 + 8);
        sh.tB = (uint32_t*)take((size_t)nwords32 * 4 + 8);
        sh.list = (uint16_t*)take((size_t)kSpListCap * 2);
        sh.accu = (double*)take((size_t)kSpThreads * 8);
        sh.accv = (double*)take((size_t)kSpThreads * 8);
        sh.red = (double*)take((size_t)kSpThreads * 8);
        sh.scal = (uint32_t*)take((size_t)2 * kSpGrid * 2 * 4);
        sh.scan = (int*)take((size_t)(kSpWaves + 1) * 4);
        pd.ps_stride = (int)mwords32 + 1;
        pd.pt_stride = (int)nwords32 + 1;
        pd.coef = (double*)take(32 * 8);
        pd.ej = (double*)take(32 * 8);
        pd.effu = (double*)take((size_t)kSpThreads * 8);
        pd.effv = (double*)take((size_t)kSpThreads * 8);
        pd.rowmask = (uint32_t*)take(16);
        pd.PS = (uint32_t*)take((size_t)width * pd.ps_stride * 4);
        pd.PT = (uint32_t*)take((size_t)width * pd.pt_stride * 4);
        pd.T0 = (uint32_t*)take((size_t)kSpAhead * pd.pt_stride * 4);
        pd.U0 = (double*)take((size_t)kSpAhead * kSpThreads * 8);
    }
    for (int64_t i = tid; i < mwords32 + 2; i += kSpThreads) {
        sh.sA[i] = 0;
        sh.sB[i] = 0;
    }
    for (int64_t i = tid; i < nwords32 + 2; i += kSpThreads) {
        sh.tA[i] = 0;
        sh.tB[i] = 0;
    }
    __syncthreads();
    uint32_t *s_cur = sh.sA, *s_oth = sh.sB, *t_cur = sh.tA, *t_oth = sh.tB;

    const int rs = a.rs, cs = a.cs;
    const int64_t i0 = (int64_t)g * rs < m ? (int64_t)g * rs : m;
    const int rlen = (int)((i0 + rs < m ? i0 + rs : m) - i0);
    const int64_t j0 = (int64_t)g * cs < n ? (int64_t)g * cs : n;
    const int clen = (int)((j0 + cs < n ? j0 + cs : n) - j0);
    TE* R = (TE*)a.R;
    TE* RT = (TE*)a.RT;
    const double total = (double)m * (double)n;

    int64_t k = a.k_start;
    uint32_t seq = a.seq;
    int alternations = 0, updates = 0, warn = 0, spins = 0;
    int64_t flips = 0, flips_rows = 0;
    int np = 0;  // pending terms
    int ahead = 0, ahead_made = 0;  // first products R' t_0 formed in advance: still unused / formed by the last pass
    uint32_t own_u = 0u, own_v = 0u;  // their signs at this thread's row of I_g / column of J_g, bit j for term j
    double F;    // ||R_k||_F^2 of the true remainder
    {
        const double f0 = a.trace[k];
        F = f0 * f0;
    }

    for (;;) {
        if (k >= a.w_target && np == 0) break;
        const bool last = k >= a.w_target;
        const bool flush = np > 0 && (np == width || last);
        // a pass over the rows of R that forms first products in advance: every flush, and the start of a launch
        // (nothing pending: the pass only reads)
        const bool pass = flush || (np == 0 && ahead == 0);
        // t_0 of term k (Algorithm 4 line 2), into the other column buffer
        for (int64_t i = tid; i < nwords32; i += kSpThreads) {
            uint32_t v = (uint32_t)(rng_word(a.seed, (uint64_t)k, 1u, (uint64_t)(i >> 1)) >> (32 * (i & 1)));
            const int64_t rem = n - i * 32;
            if (rem < 32) v &= (1u << rem) - 1u;
            t_oth[i] = v;
        }
        __syncthreads();
        double fsq = 0.0, dummy = 0.0;
        // rows I_g: u = R t_0 (Algorithm 4 line 5), from the flushed copy or from R' with the correction
        if (pass) {
            // the random starts of this term and the next ones of the launch, as many as there is room for
            const int64_t left = a.w_target - k;
            const int nvec = (int)(left < kSpAhead ? (left > 0 ? left : 0) : kSpAhead);
            for (int64_t i = tid; i < (int64_t)nvec * nwords32; i += kSpThreads) {
                const int64_t jv = i / nwords32, iw = i - jv * nwords32;
                uint32_t v = (uint32_t)(rng_word(a.seed, (uint64_t)(k + jv), 1u, (uint64_t)(iw >> 1)) >> (32 * (iw & 1)));
                const int64_t rem = n - iw * 32;
                if (rem < 32) v &= (1u << rem) - 1u;
                pd.T0[jv * pd.pt_stride + iw] = v;
            }
            __syncthreads();
            if (rlen > 0)
                sp_flush_rows<TE, kSpAhead>(R, n, i0, rlen, pd.PS, pd.ps_stride, pd.PT, pd.pt_stride, np, pd.coef, pd.T0,
                                            pd.pt_stride, nvec, pd.U0, fsq, sh.red, pd.rowmask);
            ahead = nvec;
            ahead_made = nvec;
        }
        if (pass || ahead > 0) {
            // (past the end of the launch nothing was formed and the signs published below are not used)
            const int slot = ahead > 0 ? ahead_made - ahead : 0;
            if (tid < rlen) sh.accu[tid] = pd.U0[slot * kSpThreads + tid];
            if (ahead > 0) --ahead;
        } else if (rlen > 0)
            sp_dense_rows<TE>(R, n, i0, rlen, false, s_cur, t_cur, (TE)0, t_oth, sh.accu, dummy, sh.red);
        if (flush) {
            if (tid < rlen) pd.effu[tid] = sh.accu[tid];
        } else {
            sp_pending_dots(pd.PT, pd.pt_stride, (int)nwords32, n, t_oth, np, width, pd.coef, pd.ej);
            sp_effective(sh.accu, rlen, own_u, pd.ej, width, pd.effu);
        }
        if (!sp_exchange(a, ++seq, pd.effu, rlen, rs, m, fsq, flush, s_oth, sh, spins, flush)) {
            if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
            return;
        }
        ++alternations;
        if (flush) {
            F = sp_sum_scalar(sh, sh.red, a.grid);  // measured again
            if (g == 0 && tid == 0) a.trace[k] = sqrt(F);
        }
        // rows J_g of the transposed copy: v = R^T s_1 (Algorithm 4 line 6)
        if (flush) {
            if (clen > 0)
                sp_flush_rows<TE, 1>(RT, m, j0, clen, pd.PT, pd.pt_stride, pd.PS, pd.ps_stride, np, pd.coef, s_oth, 0, 1, sh.accv,
                                     dummy, sh.red, pd.rowmask);
            updates += np;
            np = 0;
            own_u = 0u;
            own_v = 0u;
            if (last) break;
            if (tid < clen) pd.effv[tid] = sh.accv[tid];
        } else {
            if (clen > 0)
                sp_dense_rows<TE>(RT, m, j0, clen, false, t_cur, s_cur, (TE)0, s_oth, sh.accv, dummy, sh.red);
            sp_pending_dots(pd.PS, pd.ps_stride, (int)mwords32, m, s_oth, np, width, pd.coef, pd.ej);
            sp_effective(sh.accv, clen, own_v, pd.ej, width, pd.effv);
        }
        {
            uint32_t* z = s_cur; s_cur = s_oth; s_oth = z;
            z = t_cur; t_cur = t_oth; t_oth = z;
        }
        int j = 0;
        double c_prev = -INFINITY;
        bool handover = flush;  // the transposed copy was rewritten: the next exchange carries the fences
        for (;;) {
            // ---- finish the column half: t = sgn(v), c = sum |v| (Algorithm 4 lines 6-7), all-gather
            double cabs = (tid < clen) ? fabs(pd.effv[tid]) : 0.0;
            cabs = sp_wave_sum(cabs);
            __syncthreads();
            if (lane == 0) sh.red[wv] = cabs;
            __syncthreads();
            double cpart = 0.0;
            for (int q = 0; q < kSpWaves; ++q) cpart += sh.red[q];
            __syncthreads();
            if (!sp_exchange(a, ++seq, pd.effv, clen, cs, n, cpart, true, t_oth, sh, spins, handover)) {
                if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
                return;
            }
            handover = false;
            {
                uint32_t* z = t_cur; t_cur = t_oth; t_oth = z;
            }
            ++j;
            const double c = sp_sum_scalar(sh, sh.red, a.grid);
            // ---- Algorithm 4 line 8
            if (c <= c_prev || j >= a.max_iters) {
                if (!(c <= c_prev)) warn = 1;
                const double ck = c / total;
                const double ckt = (double)(TE)ck;  // the stored coefficient is what the flush subtracts
                if (g == 0) {
                    for (int p = tid; p < a.mw; p += kSpThreads)
                        a.S[k * a.mw + p] = (uint64_t)s_cur[2 * p] | ((uint64_t)(2 * p + 1 < mwords32 ? s_cur[2 * p + 1] : 0u) << 32);
                    if (tid == 0) {
                        ((TE*)a.c)[k] = (TE)ck;
                        a.iters[k] = j;
                    }
                }
                if (g == (a.grid > 1 ? 1 : 0)) {
                    for (int p = tid; p < a.nw; p += kSpThreads)
                        a.T[k * a.nw + p] = (uint64_t)t_cur[2 * p] | ((uint64_t)(2 * p + 1 < nwords32 ? t_cur[2 * p + 1] : 0u) << 32);
                }
                // the term joins the pending list (Section 3.2)
                for (int p = tid; p < (int)mwords32; p += kSpThreads) pd.PS[np * pd.ps_stride + p] = s_cur[p];
                for (int p = tid; p < (int)nwords32; p += kSpThreads) pd.PT[np * pd.pt_stride + p] = t_cur[p];
                if (tid == 0) pd.coef[np] = ckt;
                if (tid < rlen) own_u |= ((s_cur[(i0 + tid) >> 5] >> ((i0 + tid) & 31)) & 1u) << np;
                if (tid < clen) own_v |= ((t_cur[(j0 + tid) >> 5] >> ((j0 + tid) & 31)) & 1u) << np;
                __syncthreads();
                ++np;
                F = F - 2.0 * ckt * c + ckt * ckt * total;
                if (F < 0.0) F = 0.0;
                ++k;
                if (g == 0 && tid == 0) a.trace[k] = sqrt(F);
                break;
            }
            c_prev = c;
            // ---- row half, sparse: u' += 2 sum over flipped columns (rows of the transposed copy), correction, s
            sp_accumulate_flips<TE>(RT, m, i0, rlen, t_cur, t_oth, n, sh.accu, sh, flips);
            sp_pending_dots(pd.PT, pd.pt_stride, (int)nwords32, n, t_cur, np, width, pd.coef, pd.ej);
            sp_effective(sh.accu, rlen, own_u, pd.ej, width, pd.effu);
            if (!sp_exchange(a, ++seq, pd.effu, rlen, rs, m, 0.0, false, s_oth, sh, spins, false)) {
                if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
                return;
            }
            {
                uint32_t* z = s_cur; s_cur = s_oth; s_oth = z;
            }
            ++alternations;
            // ---- column half, sparse: v' += 2 sum over flipped rows, correction
            sp_accumulate_flips<TE>(R, n, j0, clen, s_cur, s_oth, m, sh.accv, sh, flips_rows);
            sp_pending_dots(pd.PS, pd.ps_stride, (int)mwords32, m, s_cur, np, width, pd.coef, pd.ej);
            sp_effective(sh.accv, clen, own_v, pd.ej, width, pd.effv);
        }
    }
    if (g == 0 && tid == 0) {
        a.res->k = k;
        a.res->alternations = alternations;
        a.res->updates = updates;
        a.res->seq_u = seq;
        a.res->seq_v = seq;
        a.res->warn = warn;
        a.res->spins = spins;
        a.res->flips = flips;
        a.res->flips_rows = flips_rows;
    }
}

// out (cols x rows) = in^T (rows x cols), 32 x 32 tiles through LDS
template <typename TE>
__global__ void __launch_bounds__(256) transpose_kernel(const TE* __restrict__ in, TE* __restrict__ out, int64_t rows,
                                                        int64_t cols)
{
    __shared__ TE tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int64_t c0 = (int64_t)blockIdx.x * 32, r0 = (int64_t)blockIdx.y * 32;
    for (int i = ty; i < 32; i += 8)
        if (r0 + i < rows && c0 + tx < cols) tile[i][tx] = in[(r0 + i) * cols + c0 + tx];
    __syncthreads();
    for (int i = ty; i < 32; i += 8)
        if (c0 + i < cols && r0 + tx < rows) out[(c0 + i) * rows + r0 + tx] = tile[tx][i];
}

size_t sparse_lds_bytes(int64_t m, int64_t n, int delay_width)
{
    auto al = [](size_t b) { return (b + 15) & ~(size_t)15; };
    const size_t mw = (size_t)((m + 31) >> 5), nw = (size_t)((n + 31) >> 5);
    size_t b = 2 * al(mw * 4 + 8) + 2 * al(nw * 4 + 8) + al((size_t)kSpListCap * 2) + 3 * al((size_t)kSpThreads * 8) +
               al((size_t)2 * kSpGrid * 2 * 4) + al((size_t)(kSpWaves + 1) * 4);
    if (delay_width > 0)
        b += 2 * al(32 * 8) + 2 * al((size_t)kSpThreads * 8) + al(16) + al((size_t)delay_width * (mw + 1) * 4) +
             al((size_t)delay_width * (nw + 1) * 4) + al((size_t)kSpAhead * (nw + 1) * 4) +
             al((size_t)kSpAhead * kSpThreads * 8);
    return b;
}

}  // namespace

bool sparse_supported(scd_dtype dt, int order, const int64_t* dims, int grid, int* rs, int* cs)
{
    if (order != 2) return false;
    if (grid < 1 || grid > kSpGrid) return false;
    const int64_t m = dims[0], n = dims[1];
    const int ve = dt == SCD_F32 ? 4 : 2;
    if (m % ve || n % ve) return false;               // rows of R and of RT start on 16-byte boundaries
    if (m > 65536 || n > 65536 || m < 8 || n < 8) return false;
    const int64_t r = 8 * ((m + 8 * grid - 1) / (8 * grid));  // slice of the rows / columns per workgroup
    const int64_t c = 8 * ((n + 8 * grid - 1) / (8 * grid));
    if (r > kSpThreads || c > kSpThreads) return false;
    if (r > 32 * kSpPayload || c > 32 * kSpPayload) return false;
    if ((int64_t)grid * (((r > c ? r : c) + 31) / 32 + 2) > (int64_t)kSpMaxItems * kSpThreads) return false;
    if (sparse_lds_bytes(m, n, 0) > kSpMaxLds) return false;
    if (rs) *rs = (int)r;
    if (cs) *cs = (int)c;
    return true;
}

size_t sparse_xbuf_bytes() { return (size_t)2 * kSpGrid * kSpSlot * 8; }

hipError_t launch_transpose(const void* in, void* out, scd_dtype dt, int64_t rows, int64_t cols, hipStream_t st)
{
    dim3 grid((unsigned)((cols + 31) / 32), (unsigned)((rows + 31) / 32));
    if (dt == SCD_F32)
        hipLaunchKernelGGL((transpose_kernel<float>), grid, dim3(256), 0, st, (const float*)in, (float*)out, rows, cols);
    else
        hipLaunchKernelGGL((transpose_kernel<double>), grid, dim3(256), 0, st, (const double*)in, (double*)out, rows, cols);
    return hipGetLastError();
}

// Most pending terms (at most 32) whose sign vectors fit into LDS beside the rest; 0 if fewer than 4 would.
int sparse_delay_width(int64_t m, int64_t n)
{
    int w = 32;
    while (w >= 4 && sparse_lds_bytes(m, n, w) > kSpMaxLds) --w;
    return w >= 4 ? w : 0;
}

template <typename TE>
static hipError_t launch_sparse_t(const SparseArgs& a, hipStream_t st)
{
    const size_t lds = sparse_lds_bytes(a.m, a.n, a.delay_width);
    if (lds > kSpMaxLds || a.delay_width < 0 || a.delay_width > 32) return hipErrorInvalidValue;
    const void* fn = a.delay_width > 0 ? (const void*)sparse_delay_kernel<TE> : (const void*)sparse_kernel<TE>;
    // always the same ceiling, whatever this launch needs: launches from several host threads set it too
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kSpMaxLds);
    if (e != hipSuccess) return e;
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess) {
        if (a.delay_width > 0) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sparse_delay_kernel<TE>, kSpThreads, lds);
        else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, sparse_kernel<TE>, kSpThreads, lds);
    }
    if (e != hipSuccess) return e;
    // all workgroups must be resident at once (every wait in the kernel is bounded in case they are not)
    if (a.grid < 1 || a.grid > kSpGrid) return hipErrorInvalidValue;
    if ((int64_t)per_cu * prop.multiProcessorCount < a.grid) return hipErrorCooperativeLaunchTooLarge;
    if (a.delay_width > 0) hipLaunchKernelGGL((sparse_delay_kernel<TE>), dim3(a.grid), dim3(kSpThreads), lds, st, a);
    else hipLaunchKernelGGL((sparse_kernel<TE>), dim3(a.grid), dim3(kSpThreads), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_sparse(const SparseArgs& a, scd_dtype dt, hipStream_t st)
{
    return dt == SCD_F32 ? launch_sparse_t<float>(a, st) : launch_sparse_t<double>(a, st);
}

}  // namespace scd
