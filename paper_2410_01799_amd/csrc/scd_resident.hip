// Probes of workgroup-to-workgroup exchange latency inside one persistent launch (measurement only).
#include "scd_device.h"
#include "scd_rng.h"

namespace scd {

__device__ __forceinline__ uint64_t tagged(float v, uint32_t tag)
{
    return ((uint64_t)tag << 32) | (uint64_t)__float_as_uint(v);
}

// Every workgroup publishes 256 tagged values per round and reads those of the `group` workgroups
// it shares a group with; value and tag travel in one 8-byte store, so the data is its own flag.
__global__ void __launch_bounds__(256) exchange_probe_kernel(uint64_t* buf, int rounds, int group, int max_spin,
                                                            unsigned* err, float* out)
{
    const int g = blockIdx.x, tid = threadIdx.x;
    const int nvals = (group >> 16) ? (group >> 16) : 256;  // values each workgroup publishes per round
    group &= 0xFFFF;
    const int g0 = (g / group) * group;
    float carry = 0.f;
    if (tid >= nvals) return;
    for (int r = 1; r <= rounds; ++r) {
        uint64_t* mine = buf + ((size_t)(r & 1) * gridDim.x + g) * 256;
        __hip_atomic_store(mine + tid, tagged(carry + (float)tid, (uint32_t)r), __ATOMIC_RELAXED,
                           __HIP_MEMORY_SCOPE_AGENT);
        float s = 0.f;
        for (int q0 = 0; q0 < group; q0 += 16) {
            // all loads of a batch of 16 members are in flight together; stale ones are retried
            uint64_t w[16];
            const int nq = group - q0 < 16 ? group - q0 : 16;
            unsigned pending = (nq == 16) ? 0xFFFFu : ((1u << nq) - 1u);
            int spin = 0;
            while (pending) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const uint64_t* theirs = buf + ((size_t)(r & 1) * gridDim.x + g0 + q0 + (q < nq ? q : 0)) * 256;
                    if ((pending >> q) & 1u)
                        w[q] = __hip_atomic_load(theirs + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int q = 0; q < 16; ++q)
                    if (((pending >> q) & 1u) && (uint32_t)(w[q] >> 32) == (uint32_t)r) pending &= ~(1u << q);
                if (pending && ++spin > max_spin) {
                    atomicExch(err, 1u);
                    return;
                }
            }
#pragma unroll
            for (int q = 0; q < 16; ++q)
                if (q < nq) s += __uint_as_float((uint32_t)w[q]);
        }
        carry = s * 1e-3f;
    }
    if (tid == 0) out[g] = carry;
}

// Classic counter barrier over the whole grid, for comparison.
__global__ void __launch_bounds__(256) barrier_probe_kernel(unsigned* counter, int rounds, int max_spin, unsigned* err,
                                                           float* out)
{
    unsigned target = 0;
    for (int r = 1; r <= rounds; ++r) {
        __syncthreads();
        if (threadIdx.x == 0) {
            __threadfence();
            __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            target += gridDim.x;
            int spin = 0;
            while (__hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (++spin > max_spin) {
                    atomicExch(err, 1u);
                    break;
                }
                __builtin_amdgcn_s_sleep(1);
            }
            __threadfence();
        }
        __syncthreads();
        if (*(volatile unsigned*)err) return;
    }
    if (threadIdx.x == 0) out[blockIdx.x] = (float)target;
}

hipError_t launch_exchange_probe(int which, int grid, uint64_t* buf, unsigned* counter, int rounds, int group,
                                 int max_spin, unsigned* err, float* out, hipStream_t st)
{
    if (which == 0)
        hipLaunchKernelGGL(exchange_probe_kernel, dim3(grid), dim3(256), 0, st, buf, rounds, group, max_spin, err, out);
    else
        hipLaunchKernelGGL(barrier_probe_kernel, dim3(grid), dim3(256), 0, st, counter, rounds, max_spin, err, out);
    return hipGetLastError();
}

// ---- helpers of the engine

// Sum over the 64 lanes, the same bits in every lane, without LDS traffic (a chain of ds_bpermute would cost
// an LDS round trip per step): distances 1, 2, 4, 8 by the data-parallel lane modes (4 = mirror of half a row
// then reversed quads, 8 = mirror of a row then of half a row), 16 and 32 by the row-swap instructions of
// gfx950 (swapping the odd rows of one copy with the even rows of another leaves the two partners of every
// lane in the two results, in the same order for both partners).
template <int C0, int C1>
__device__ __forceinline__ double dpp_f64_res(double v)
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
__device__ __forceinline__ double swap_sum_f64_res(double a)
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
__device__ __forceinline__ double wave_sum_res(double a)
{
    a += dpp_f64_res<0xB1, 0>(a);       // lane ^ 1
    a += dpp_f64_res<0x4E, 0>(a);       // lane ^ 2
    a += dpp_f64_res<0x141, 0x1B>(a);   // lane ^ 4
    a += dpp_f64_res<0x140, 0x141>(a);  // lane ^ 8
    a = swap_sum_f64_res<16>(a);
    a = swap_sum_f64_res<32>(a);
    return a;
}


// =================================================================================================
// Register-resident engine.
//
// A 4096 x 4096 f32 remainder is 64 MiB; the 256 compute units of the chip hold 128 MiB of vector
// registers.  Workgroup (pr, pc) of a 16 x 16 grid keeps block (pr, pc) of R in its registers for the
// whole run, so an alternation of Algorithm 4 moves no matrix data at all: only 256 partial sums per
// workgroup and phase travel through memory.
//
//   row phase   p_i = sum over the block's columns of +-R_il (signs t), published to the 16
//               workgroups of the same block row; each adds the 16 partials in order -> u_i, s_i
//   col phase   q_l = sum over the block's rows of +-R_il (signs s), published to the 16 workgroups
//               of the same block column -> v_l, t_l, and this column block's share of c = sum |v_l|
//
// Exchange: value and sequence number travel in one 8-byte store (the datum is its own flag), read
// back with loads that bypass the non-coherent caches; no counter, no fence.  Slots alternate by the
// parity of the sequence number: a workgroup can only be one exchange ahead of the readers of its
// slot, because finishing exchange e+1 needs data its readers publish after they have read e.
// The sum of the 16 column-block shares of c rides on the next row-phase exchange, so the test of
// Algorithm 4 line 8 is taken one phase late: the row phase already done with the final t is then
// dropped.  ||R||_F^2 after an update travels the same way (block row sums, then the total).
// Every wait is bounded; on expiry all workgroups leave and the host reports an error.

// word offset of the slot of workgroup `wg` for exchange `seq` of kind 0 (rows) or 1 (columns)
__device__ __forceinline__ uint32_t res_slot_off(int kind, uint32_t seq, int wg)
{
    return (uint32_t)(((kind * 2 + (int)(seq & 1u)) * (kResGrid * kResGrid) + wg) * kResSlotWords);
}
__device__ __forceinline__ uint64_t* res_slot(const ResidentArgs& a, int kind, uint32_t seq, int wg)
{
    return a.xbuf + res_slot_off(kind, seq, wg);
}

__device__ __forceinline__ double uniform_f64(double v)
{
    // the value is the same in every lane: keep it in scalar registers
    const long long b = __double_as_longlong(v);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(b & 0xFFFFFFFFll));
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

__device__ __forceinline__ void res_publish(uint64_t* p, float v, uint32_t seq)
{
    __hip_atomic_store(p, ((uint64_t)seq << 32) | (uint64_t)__float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ void res_publish_f64(uint64_t* p, double v, uint32_t seq)
{
    const uint64_t b = (uint64_t)__double_as_longlong(v);
    __hip_atomic_store(p, ((uint64_t)seq << 32) | (b & 0xFFFFFFFFull), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(p + 1, ((uint64_t)seq << 32) | (b >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// H members' values of one element (one half of a group of 2H) plus NX / 2 piggybacked doubles of one
// member (NX = 2 or 4 more words; only what the phase at hand uses is published and read: every word is a
// trip through the fabric), all loads in flight together.  If any word is still from an earlier exchange,
// all are read again (re-reads are rare once the first read is delayed a little).
template <int H, int NX>
__device__ __forceinline__ bool res_gather_x2(const uint64_t* xbuf, uint32_t off, uint32_t stride, uint32_t xoff,
                                              uint32_t seq, int max_spin, double& sum, double& x0, double& x1,
                                              int& spin)
{
    static_assert(NX == 2 || NX == 4, "one or two piggybacked doubles");
    uint64_t w[H + 4];
    w[H + 2] = 0;
    w[H + 3] = 0;
    for (;;) {
#pragma unroll
        for (int q = 0; q < H; ++q)
            w[q] = __hip_atomic_load(xbuf + (off + q * stride), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
        for (int q = 0; q < NX; ++q)
            w[H + q] = __hip_atomic_load(xbuf + (xoff + q), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool fresh = true;
#pragma unroll
        for (int q = 0; q < H + NX; ++q) fresh = fresh && ((uint32_t)(w[q] >> 32) == seq);
        if (fresh) break;
        if (++spin > max_spin) return false;
        __builtin_amdgcn_s_sleep(1);
    }
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < H; ++q) s += (double)__uint_as_float((uint32_t)w[q]);
    sum = s;
    x0 = __longlong_as_double((long long)((w[H + 1] << 32) | (w[H] & 0xFFFFFFFFull)));
    x1 = __longlong_as_double((long long)((w[H + 3] << 32) | (w[H + 2] & 0xFFFFFFFFull)));
    return true;
}

// H members' values of one element, all loads in flight together.
template <int H>
__device__ __forceinline__ bool res_gather(const uint64_t* xbuf, uint32_t off, uint32_t stride, uint32_t seq,
                                           int max_spin, double& sum, int& spin)
{
    uint64_t w[H];
    for (;;) {
#pragma unroll
        for (int q = 0; q < H; ++q)
            w[q] = __hip_atomic_load(xbuf + (off + q * stride), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        bool fresh = true;
#pragma unroll
        for (int q = 0; q < H; ++q) fresh = fresh && ((uint32_t)(w[q] >> 32) == seq);
        if (fresh) break;
        if (++spin > max_spin) return false;
        __builtin_amdgcn_s_sleep(1);
    }
    double s = 0.0;
#pragma unroll
    for (int q = 0; q < H; ++q) s += (double)__uint_as_float((uint32_t)w[q]);
    sum = s;
    return true;
}

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}

// the value of the neighbouring lane (lane ^ 1), for doubles
__device__ __forceinline__ double dpp_swap1_f64(double v)
{
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xFFFFFFFFll), 0xB1, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), 0xB1, 0xF, 0xF, true);
    return __longlong_as_double(((long long)hi << 32) | (long long)(unsigned)lo);
}

// v[l] + v[l ^ 16] and v[l] + v[l ^ 32] by the row-swap instructions of gfx950 (no LDS traffic):
// swapping the odd rows of one copy with the even rows of another leaves the two partners of every
// lane in the two results, in the same order for both partners.
__device__ __forceinline__ float sum_xor16(float v)
{
    const unsigned b = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane16_swap(b, b, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
__device__ __forceinline__ float sum_xor32(float v)
{
    const unsigned b = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// PAD: the grid overhangs the matrix (a template parameter: the 128 row/column tests of a thread's tile are
// invariants of the whole launch, and a kernel that has to keep them takes twice the instructions and runs out of
// scalar registers even when no test ever fails).
template <int TR, int TC, int P, bool PAD>
__global__ void __launch_bounds__(kResThreads) resident_kernel(ResidentArgs a)
{
    constexpr int H = P / 2;  // members per half of an exchange group
    static_assert(P == 4 || P == 8 || P == 16, "grid side");
    constexpr int BM = 32 * TR, BN = 16 * TC;  // block of this workgroup
    static_assert(TR >= 2 && TR <= 16 && (TR % 2) == 0, "rows per thread");
    static_assert(TC >= 4 && TC <= 32 && (TC % 4) == 0, "columns per thread");
    static_assert(BM + 4 <= kResSlotWords && BN + 4 <= kResSlotWords, "slot size");
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int tr = tid >> 4, tc = tid & 15;  // 32 x 16 threads, each TR x TC elements
    const int pr = blockIdx.x / P, pc = blockIdx.x % P;
    const int wg = blockIdx.x;

    __shared__ float lds_q[kResThreads / 64][BN];
    __shared__ uint8_t lds_s[2][BM];
    __shared__ uint8_t lds_t[BN];
    __shared__ double lds_red[kResThreads / 64];
    __shared__ double lds_x[2][P];

    // ---- load the block.  The grid may overhang the matrix: rows and columns past its end are zeros in the
    // registers (they add nothing to any sum and stay zero through every update) and are never read or written.
    const int64_t row0 = (int64_t)pr * BM + tr * TR, col0 = (int64_t)pc * BN + tc * TC;
    constexpr bool padded = PAD;
    float x[TR][TC];
    {
        const float* base = a.R + row0 * a.n + col0;
#pragma unroll
        for (int r = 0; r < TR; ++r)
#pragma unroll
            for (int c4 = 0; c4 < TC / 4; ++c4) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (!padded || (row0 + r < a.m && col0 + 4 * c4 < a.n)) v = *(const float4*)(base + (int64_t)r * a.n + 4 * c4);
                x[r][4 * c4 + 0] = v.x;
                x[r][4 * c4 + 1] = v.y;
                x[r][4 * c4 + 2] = v.z;
                x[r][4 * c4 + 3] = v.w;
            }
    }

    int64_t k = a.k_start;
    int alternations = 0, updates = 0;
    uint32_t seq_u = a.seq_u, seq_v = a.seq_v;
    int j = 0, warn = 0, cur = 0;
    double c_prev = -INFINITY;
    double cpart = 0.0;      // this column block's sum |v_l| of the last column phase
    double fsq_block = 0.0;  // sum of squares of this block after the last update
    double frow = 0.0;       // ... of this block row
    int norm_stage = 0;      // 1: fsq_block to publish (row exchange); 2: frow to publish (col exchange)
    int64_t norm_k = 0;
    const double total = (double)a.m * (double)a.n;
    bool need_t0 = true;
    int spin = 0, spins = 0;

    for (;;) {
        if (k >= a.w_target && norm_stage == 0) break;
        if (need_t0) {
            // t_0 of term k from the keyed stream (Algorithm 4 line 2)
            if (tid < BN) {
                const int64_t col = (int64_t)pc * BN + tid;
                lds_t[tid] = col < a.n ? (uint8_t)((rng_word(a.seed, (uint64_t)k, 1u, (uint64_t)(col >> 6)) >> (col & 63)) & 1ull) : 0;
            }
            need_t0 = false;
            __syncthreads();
        }
        // ================= row phase: u = R t (Algorithm 4 line 5)
        // The signs enter as +-1.0 multipliers of a fused multiply-add: x * (+-1) is exact, so each step
        // rounds exactly like the sign-flip-and-add of Section 3.4, in one instruction instead of two
        // (this engine is bound by vector instructions and latency, not by memory).
        float tf[TC];
#pragma unroll
        for (int c = 0; c < TC; ++c) tf[c] = __uint_as_float(0x3F800000u | ((uint32_t)lds_t[tc * TC + c] << 31));
        float p[TR];
#pragma unroll
        for (int r = 0; r < TR; ++r) {
            float s = 0.f;
#pragma unroll
            for (int c = 0; c < TC; ++c) s = __builtin_fmaf(x[r][c], tf[c], s);
            // sum over the 16 lanes that share these rows (fixed order per lane)
            s += dpp_f32<0xB1>(s);   // lane ^ 1
            s += dpp_f32<0x4E>(s);   // lane ^ 2
            s += dpp_f32<0x124>(s);  // row rotate 4
            s += dpp_f32<0x128>(s);  // row rotate 8
            p[r] = s;
        }
        ++seq_u;
        ++alternations;
        {
            uint64_t* mine = res_slot(a, 0, seq_u, wg);
            if (tc < TR) {
                float v = p[0];
#pragma unroll
                for (int r = 1; r < TR; ++r) v = (tc == r) ? p[r] : v;
                res_publish(mine + tr * TR + tc, v, seq_u);
            }
            if (tid == 0) {
                res_publish_f64(mine + BM, cpart, seq_u);
                if (norm_stage == 1) res_publish_f64(mine + BM + 2, fsq_block, seq_u);  // (only the exchange after an update)
            }
        }
        for (int d = 0; d < a.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
        bool ok = true;
        {
            // gather: thread (row, half) adds eight members in order, the two halves are combined low
            // first.  The last wave also fetches the piggybacked scalars (lane mod P = member), in the
            // same batch of loads; threads past the block's rows read a valid row and drop it.
            const int row = tid >> 1, h = tid & 1;
            const int rowc = row < BM ? row : BM - 1;
            const uint32_t off = res_slot_off(0, seq_u, pr * P + h * H) + (uint32_t)rowc;
            double half = 0.0;
            if (wv == kResThreads / 64 - 1) {
                double x0 = 0.0, x1 = 0.0;
                const uint32_t xoff = res_slot_off(0, seq_u, pr * P + (lane & (P - 1))) + BM;
                if (norm_stage == 1) ok = res_gather_x2<H, 4>(a.xbuf, off, kResSlotWords, xoff, seq_u, a.max_spin, half, x0, x1, spin);
                else ok = res_gather_x2<H, 2>(a.xbuf, off, kResSlotWords, xoff, seq_u, a.max_spin, half, x0, x1, spin);
                if (lane < P) {
                    lds_x[0][lane] = x0;
                    lds_x[1][lane] = x1;
                }
            } else {
                ok = res_gather<H>(a.xbuf, off, kResSlotWords, seq_u, a.max_spin, half, spin);
            }
            const double other = dpp_swap1_f64(half);
            const double u = h ? other + half : half + other;
            if (h == 0 && row < BM) lds_s[cur ^ 1][row] = (u < 0.0) ? 1 : 0;
        }
        if (__syncthreads_or(ok ? 0 : 1)) {
            if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
            return;
        }
        spins += spin;
        spin = 0;
        // (all loads first, then the adds in order: a dependent chain of LDS reads would cost a latency each)
        double c_tot = 0.0;
        {
            double cq[P];
#pragma unroll
            for (int q = 0; q < P; ++q) cq[q] = lds_x[0][q];
#pragma unroll
            for (int q = 0; q < P; ++q) c_tot += cq[q];
        }
        c_tot = uniform_f64(c_tot);
        if (norm_stage == 1) {
            double f_tot = 0.0;
            double fq[P];
#pragma unroll
            for (int q = 0; q < P; ++q) fq[q] = lds_x[1][q];
#pragma unroll
            for (int q = 0; q < P; ++q) f_tot += fq[q];
            frow = uniform_f64(f_tot);
            norm_stage = 2;
        }
        if (j > 0) {
            const bool conv = (c_tot <= c_prev) || (j >= a.max_iters);
            if (conv) {
                // ---- the term is (c_tot, s_cur, t): append it (Algorithm 5 lines 7-9) and subtract it (line 10)
                if (!(c_tot <= c_prev)) warn = 1;
                const double ck = c_tot / total;
                const float ckf = (float)ck;
                if (pc == 0 && wv < BM / 64) {
                    const uint64_t word = __ballot(lds_s[cur][wv * 64 + lane] != 0);
                    if (lane == 0 && pr * (BM / 64) + wv < a.mw) a.S[k * a.mw + pr * (BM / 64) + wv] = word;
                }
                if (pr == 0 && wv < BN / 64) {
                    const uint64_t word = __ballot(lds_t[wv * 64 + lane] != 0);
                    if (lane == 0 && pc * (BN / 64) + wv < a.nw) a.T[k * a.nw + pc * (BN / 64) + wv] = word;
                }
                if (wg == 0 && tid == 0) {
                    a.c[k] = ckf;
                    a.iters[k] = j;
                }
                double f = 0.0;
#pragma unroll
                for (int r = 0; r < TR; ++r) {
                    const uint32_t sr = (uint32_t)lds_s[cur][tr * TR + r] << 31;
#pragma unroll
                    for (int c = 0; c < TC; ++c) {
                        // R_il - ck s_i t_l: the signs choose +ck or -ck
                        const float d = __uint_as_float(__float_as_uint(ckf) ^ sr ^ (__float_as_uint(tf[c]) & 0x80000000u));
                        x[r][c] = (!padded || (row0 + r < a.m && col0 + c < a.n)) ? x[r][c] - d : 0.f;  // padding stays zero
                        f += (double)x[r][c] * (double)x[r][c];
                    }
                }
                f = wave_sum_res(f);
                if (lane == 0) lds_red[wv] = f;
                __syncthreads();
                double fb = 0.0;
#pragma unroll 2
                for (int q = 0; q < kResThreads / 64; ++q) fb += lds_red[q];
                fsq_block = uniform_f64(fb);
                ++k;
                ++updates;
                norm_stage = 1;
                norm_k = k;
                j = 0;
                c_prev = -INFINITY;
                cpart = 0.0;
                need_t0 = true;
                __syncthreads();  // lds_t and lds_red are rewritten next
                continue;
            }
            c_prev = c_tot;
        }
        cur ^= 1;  // s_j = sgn(u)

        // ================= column phase: v = R^T s (Algorithm 4 line 6), c = sum |v| (line 7)
        {
            float sf[TR];
#pragma unroll
            for (int r = 0; r < TR; ++r) sf[r] = __uint_as_float(0x3F800000u | ((uint32_t)lds_s[cur][tr * TR + r] << 31));
#pragma unroll
            for (int c4 = 0; c4 < TC / 4; ++c4) {
                float qv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float s = 0.f;
#pragma unroll
                    for (int r = 0; r < TR; ++r) s = __builtin_fmaf(x[r][4 * c4 + e], sf[r], s);
                    // the four thread rows of this wave hold the same columns 16 lanes apart
                    qv[e] = sum_xor32(sum_xor16(s));
                }
                if (lane < 16) *(float4*)&lds_q[wv][tc * TC + 4 * c4] = make_float4(qv[0], qv[1], qv[2], qv[3]);
            }
        }
        __syncthreads();
        ++seq_v;
        {
            uint64_t* mine = res_slot(a, 1, seq_v, wg);
            if (tid < BN) {
                float s = 0.f;
#pragma unroll
                for (int q = 0; q < kResThreads / 64; ++q) s += lds_q[q][tid];
                res_publish(mine + tid, s, seq_v);
            }
            if (norm_stage == 2 && tid == kResThreads - 1) res_publish_f64(mine + BN, frow, seq_v);
        }
        for (int d = 0; d < a.poll_delay; ++d) __builtin_amdgcn_s_sleep(1);
        ok = true;
        double absv = 0.0;
        {
            const int col = tid >> 1, h = tid & 1;
            const int colc = col < BN ? col : BN - 1;
            const uint32_t off = res_slot_off(1, seq_v, (h * H) * P + pc) + (uint32_t)colc;
            double half = 0.0;
            if (norm_stage == 2 && wv == kResThreads / 64 - 1) {
                // the block-row sums of squares travel on this exchange once per term
                double x0 = 0.0, x1 = 0.0;
                ok = res_gather_x2<H, 2>(a.xbuf, off, P * kResSlotWords, res_slot_off(1, seq_v, (lane & (P - 1)) * P + pc) + BN,
                                         seq_v, a.max_spin, half, x0, x1, spin);
                if (lane < P) lds_x[1][lane] = x0;
            } else {
                ok = res_gather<H>(a.xbuf, off, P * kResSlotWords, seq_v, a.max_spin, half, spin);
            }
            const double other = dpp_swap1_f64(half);
            const double v = h ? other + half : half + other;
            if (h == 0 && col < BN) {
                lds_t[col] = (v < 0.0) ? 1 : 0;
                absv = fabs(v);
            }
        }
        absv = wave_sum_res(absv);
        if (lane == 0) lds_red[wv] = absv;
        if (__syncthreads_or(ok ? 0 : 1)) {
            if (tid == 0) atomicExch((unsigned*)&a.res->err, 1u);
            return;
        }
        {
            double cs = 0.0;
            {
                double cq[kResThreads / 64];
#pragma unroll
                for (int q = 0; q < kResThreads / 64; ++q) cq[q] = lds_red[q];
#pragma unroll
                for (int q = 0; q < kResThreads / 64; ++q) cs += cq[q];
            }
            cpart = uniform_f64(cs);
            if (norm_stage == 2) {
                double ft = 0.0;
                double fq[P];
#pragma unroll
                for (int q = 0; q < P; ++q) fq[q] = lds_x[1][q];
#pragma unroll
                for (int q = 0; q < P; ++q) ft += fq[q];
                ft = uniform_f64(ft);
                if (wg == 0 && tid == 0) a.trace[norm_k] = sqrt(ft);
                norm_stage = 0;
            }
        }
        ++j;
        spins += spin;
        spin = 0;
        // No barrier here: what was read above (lds_red, lds_x[1]) is next written after the two barriers of the
        // coming row and column phases (lds_x[1] in a row phase only right after an update, never right after
        // the column phase that read it), and what the coming row phase writes first (lds_s of the other
        // parity, lds_x[0]) was last read before this phase's barriers.
    }

    // ---- write the block back
    {
        float* base = a.R + row0 * a.n + col0;
#pragma unroll
        for (int r = 0; r < TR; ++r)
#pragma unroll
            for (int c4 = 0; c4 < TC / 4; ++c4)
                if (!padded || (row0 + r < a.m && col0 + 4 * c4 < a.n))
                    *(float4*)(base + (int64_t)r * a.n + 4 * c4) =
                        make_float4(x[r][4 * c4], x[r][4 * c4 + 1], x[r][4 * c4 + 2], x[r][4 * c4 + 3]);
    }
    if (wg == 0 && tid == 0) {
        a.res->k = k;
        a.res->alternations = alternations;
        a.res->updates = updates;
        a.res->seq_u = seq_u;
        a.res->seq_v = seq_v;
        a.res->warn = warn;
        a.res->spins = spins;
    }
}

// Grid side P and thread tile TR x TC for an m x n matrix: the P x P workgroups of 32 x 16 threads cover
// P * 32 * TR rows and P * 16 * TC columns, at least the matrix (the overhang is kept as zeros).  Fewer
// workgroups mean fewer partners per exchange, more workgroups less arithmetic each; measured on the square
// sizes (256 and 512 fastest with 8 values per thread on 4 x 4 and 8 x 8 workgroups, 1024 with 32 values on
// 8 x 8, 2048 with 32 values on 16 x 16), which gives the order of preference: the smallest grid of at most
// 8 x 8 with at most 8 values per thread, else the smallest grid with at most 32, else the grid that fits with
// the smallest tile.  Rows must be a multiple of 16 bytes.
static bool resident_shape(int64_t m, int64_t n, int* p, int* tr, int* tc)
{
    if (m < 1 || n < 4 || (n % 4)) return false;
    static const int grids[3] = {4, 8, 16};
    static const int trs[3] = {2, 4, 8}, tcs[3] = {4, 8, 16};
    int best = -1, bp = 0, btr = 0, btc = 0;
    for (int pass = 0; pass < 2; ++pass) {
        for (int P : grids) {
            int r = 0, c = 0;
            for (int t : trs)
                if (!r && (int64_t)P * 32 * t >= m) r = t;
            for (int t : tcs)
                if (!c && (int64_t)P * 16 * t >= n) c = t;
            if (!r || !c) continue;
            if (P == 4 && r * c > 32) continue;  // (the 4 x 4 grid is built with the small tiles only)
            if (pass == 0 ? (P <= 8 && r * c <= 8) : (r * c <= 32)) {
                *p = P, *tr = r, *tc = c;
                return true;
            }
            if (best < 0 || r * c < best) best = r * c, bp = P, btr = r, btc = c;
        }
    }
    if (best < 0) return false;
    *p = bp, *tr = btr, *tc = btc;
    return true;
}

bool resident_supported(scd_dtype dt, int order, const int64_t* dims)
{
    int p, tr, tc;
    return dt == SCD_F32 && order == 2 && resident_shape(dims[0], dims[1], &p, &tr, &tc);
}

int resident_workgroups(const int64_t* dims)
{
    int p = 0, tr, tc;
    return resident_shape(dims[0], dims[1], &p, &tr, &tc) ? p * p : 0;
}

template <int TR, int TC, int P, bool PAD>
static hipError_t launch_resident_k(const ResidentArgs& a, hipStream_t st)
{
    // All P x P workgroups must be resident at once.  One workgroup of 512 threads fits every compute
    // unit (checked here against the occupancy the runtime reports); an ordinary launch on an idle
    // device then places them all, and every wait in the kernel is bounded in case it does not.
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipGetDeviceProperties(&prop, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, resident_kernel<TR, TC, P, PAD>, kResThreads, 0);
    if (e != hipSuccess) return e;
    if ((int64_t)per_cu * prop.multiProcessorCount < P * P) return hipErrorCooperativeLaunchTooLarge;
    hipLaunchKernelGGL((resident_kernel<TR, TC, P, PAD>), dim3(P * P), dim3(kResThreads), 0, st, a);
    return hipGetLastError();
}

template <int TR, int TC, int P>
static hipError_t launch_resident_t(const ResidentArgs& a, hipStream_t st)
{
    // does the grid of P x P blocks of 32 TR x 16 TC overhang the matrix?
    const bool padded = (int64_t)P * 32 * TR != a.m || (int64_t)P * 16 * TC != a.n;
    return padded ? launch_resident_k<TR, TC, P, true>(a, st) : launch_resident_k<TR, TC, P, false>(a, st);
}

template <int P>
static hipError_t launch_resident_p(const ResidentArgs& a, int tr, int tc, hipStream_t st)
{
    const int key = tr * 100 + tc;
    switch (key) {
        case 204: return launch_resident_t<2, 4, P>(a, st);
        case 208: return launch_resident_t<2, 8, P>(a, st);
        case 404: return launch_resident_t<4, 4, P>(a, st);
        case 408: return launch_resident_t<4, 8, P>(a, st);
        default: break;
    }
    if constexpr (P >= 8) {
        switch (key) {
            case 216: return launch_resident_t<2, 16, P>(a, st);
            case 416: return launch_resident_t<4, 16, P>(a, st);
            case 804: return launch_resident_t<8, 4, P>(a, st);
            case 808: return launch_resident_t<8, 8, P>(a, st);
            case 816: return launch_resident_t<8, 16, P>(a, st);
            default: break;
        }
    }
    return hipErrorInvalidValue;
}

hipError_t launch_resident(const ResidentArgs& a, hipStream_t st)
{
    int p = 0, tr = 0, tc = 0;
    if (!resident_shape(a.m, a.n, &p, &tr, &tc)) return hipErrorInvalidValue;
    if (p == 16) return launch_resident_p<16>(a, tr, tc, st);
    if (p == 8) return launch_resident_p<8>(a, tr, tc, st);
    return launch_resident_p<4>(a, tr, tc, st);
}

}  // namespace scd
