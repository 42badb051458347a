// Product of a signed cut decomposition with a vector, straight from the packed factors
// (Section 6.1 of arXiv 2410.01799, Question A):
//     y = (sum_j c_j s_j t_j^T) x = sum_j z_j s_j,    z_j = c_j <t_j, x>.
// The matrix is never expanded: the kernels read the w (m + n) / 8 bytes of sign bits once and do one
// select and one add per bit.
//
// f32: both passes are contractions of a +-1 matrix with a vector and run on the matrix cores in block
// fixed point (see the two MFMA kernels).  f64: vector units; a wave owns 64 consecutive entries (one per
// lane), takes a 64-bit word of sign bits that is the same for all its lanes (fetched by one lane,
// broadcast through a scalar register), turns bit `lane` into a multiplier +-1.0 and adds with one fused
// multiply-add in f64 (the product with +-1 is exact, so each step rounds like the sign-flip-and-add of
// Section 3.4).
//   inner pass  <t_j, x> per chunk of 4096 entries
//   outer pass  z_j = c_j * (sum of the chunk parts, in order) is formed on the way in; per split of the
//               terms, y_i = sum_j +-z_j
//   reduce      y = sum of the splits, in order, rounded once to the output type
// Every sum has a fixed order: results are bit-identical from run to run.
#include "scd_device.h"

namespace scd {

namespace {

constexpr int kApChunkWords = 64;   // words of sign bits per lane-resident chunk of x (4096 entries)
constexpr int kApInnerWaves = 4;    // waves per workgroup of the inner pass
constexpr int kApOuterWaves = 8;    // waves per workgroup of the outer pass: 8 adjacent words = one 64-byte line

// Cross-lane steps without LDS traffic (a chain of ds_bpermute costs an LDS round trip per step): the value
// of lane (l ^ D) for D = 1, 2, 4, 8 by the data-parallel lane modes (4 = mirror of half a row then reversed
// quads, 8 = mirror of a row then of half a row); the two partners at distance 16 or 32 by the row-swap
// instructions of gfx950 (swapping the odd rows of one copy with the even rows of another leaves them in the
// two results, in the same order for both partners).
template <int D>
__device__ __forceinline__ uint32_t ap_dpp_xor(uint32_t v)
{
    static_assert(D == 1 || D == 2 || D == 4 || D == 8, "distance within a row of 16 lanes");
    constexpr int c0 = D == 1 ? 0xB1 : D == 2 ? 0x4E : D == 4 ? 0x141 : 0x140;
    constexpr int c1 = D == 4 ? 0x1B : D == 8 ? 0x141 : 0;
    int r = __builtin_amdgcn_update_dpp(0, (int)v, c0, 0xF, 0xF, true);
    if constexpr (c1 != 0) r = __builtin_amdgcn_update_dpp(0, r, c1, 0xF, 0xF, true);
    return (uint32_t)r;
}
template <int D>
__device__ __forceinline__ double ap_dpp_xor_f64(double v)
{
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    const uint32_t lo = ap_dpp_xor<D>((uint32_t)b), hi = ap_dpp_xor<D>((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// (a, b) = the values of the two partners at distance D = 16 or 32, the same pair in both of them
template <int D>
__device__ __forceinline__ void ap_swap_pair(uint32_t v, uint32_t& a, uint32_t& b)
{
    if constexpr (D == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        a = r[0], b = r[1];
    } else {
        const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        a = r[0], b = r[1];
    }
}
template <int D>
__device__ __forceinline__ void ap_swap_pair_f64(double v, double& a, double& b)
{
    const unsigned long long w = (unsigned long long)__double_as_longlong(v);
    uint32_t la, lb, ha, hb;
    ap_swap_pair<D>((uint32_t)w, la, lb);
    ap_swap_pair<D>((uint32_t)(w >> 32), ha, hb);
    a = __longlong_as_double((long long)(((unsigned long long)ha << 32) | la));
    b = __longlong_as_double((long long)(((unsigned long long)hb << 32) | lb));
}

__device__ __forceinline__ double ap_wave_sum(double a)
{
    a += ap_dpp_xor_f64<1>(a);
    a += ap_dpp_xor_f64<2>(a);
    a += ap_dpp_xor_f64<4>(a);
    a += ap_dpp_xor_f64<8>(a);
    double p, q;
    ap_swap_pair_f64<16>(a, p, q);
    a = p + q;
    ap_swap_pair_f64<32>(a, p, q);
    return p + q;
}
__device__ __forceinline__ double ap_wave_max(double a)
{
    a = fmax(a, ap_dpp_xor_f64<1>(a));
    a = fmax(a, ap_dpp_xor_f64<2>(a));
    a = fmax(a, ap_dpp_xor_f64<4>(a));
    a = fmax(a, ap_dpp_xor_f64<8>(a));
    double p, q;
    ap_swap_pair_f64<16>(a, p, q);
    a = fmax(p, q);
    ap_swap_pair_f64<32>(a, p, q);
    return fmax(p, q);
}
__device__ __forceinline__ float ap_wave_max(float a)
{
    a = fmaxf(a, __uint_as_float(ap_dpp_xor<1>(__float_as_uint(a))));
    a = fmaxf(a, __uint_as_float(ap_dpp_xor<2>(__float_as_uint(a))));
    a = fmaxf(a, __uint_as_float(ap_dpp_xor<4>(__float_as_uint(a))));
    a = fmaxf(a, __uint_as_float(ap_dpp_xor<8>(__float_as_uint(a))));
    uint32_t p, q;
    ap_swap_pair<16>(__float_as_uint(a), p, q);
    a = fmaxf(__uint_as_float(p), __uint_as_float(q));
    ap_swap_pair<32>(__float_as_uint(a), p, q);
    return fmaxf(__uint_as_float(p), __uint_as_float(q));
}

// +-1.0 for lane `lane` from bit `lane` of a wave-uniform word (a 1 bit stands for -1)
__device__ __forceinline__ double ap_sign(uint64_t word)
{
    const int hi = __builtin_amdgcn_inverse_ballot_w64(word) ? (int)0xBFF00000 : (int)0x3FF00000;
    return __hiloint2double(hi, 0);
}

// word `p` of a lane-distributed row of sign bits (lane p holds word p), as a wave-uniform value
__device__ __forceinline__ uint64_t ap_word(uint64_t lane_word, int p)
{
    const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)lane_word, p);
    const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)(lane_word >> 32), p);
    return ((uint64_t)hi << 32) | lo;
}

constexpr int kApDepth = 4;  // rows of sign bits in flight per wave

template <typename TE>
__global__ void __launch_bounds__(kApInnerWaves* kWave)
    apply_inner_kernel(const uint64_t* __restrict__ bits, int64_t nw, int64_t w, const TE* __restrict__ x, int64_t n,
                       double* __restrict__ part, int terms_per_wave)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t chunk = blockIdx.y;
    const int64_t p0 = chunk * kApChunkWords;
    const int nwc = (int)(nw - p0 < kApChunkWords ? nw - p0 : kApChunkWords);  // words of this chunk
    double xr[kApChunkWords];
#pragma unroll
    for (int p = 0; p < kApChunkWords; ++p) {
        // unconditional loads (all in flight together); entries past the end count as zero
        const int64_t l = (p0 + p) * 64 + lane;
        const TE v = x[l < n ? l : n - 1];
        xr[p] = l < n ? (double)v : 0.0;
    }
    const int64_t j0 = ((int64_t)blockIdx.x * kApInnerWaves + wv) * terms_per_wave;
    const int64_t j1 = j0 + terms_per_wave < w ? j0 + terms_per_wave : w;
    if (j0 >= j1) return;
    // Lane p fetches word p of a term's row (one coalesced load per term), kApDepth terms ahead.  Loads
    // are unconditional: terms past the end re-read the last one, lanes past the end of the row read its
    // first word (the entries of x there are zero, so any valid word will do).
    const int64_t lw = p0 + (lane < nwc ? lane : 0);
    uint64_t buf[kApDepth];
#pragma unroll
    for (int d = 0; d < kApDepth; ++d) {
        const int64_t jn = j0 + d < j1 ? j0 + d : j1 - 1;
        buf[d] = bits[jn * nw + lw];
    }
    for (int64_t j = j0; j < j1; j += kApDepth) {
#pragma unroll
        for (int d = 0; d < kApDepth; ++d) {
            const uint64_t row = buf[d];
            const int64_t jn = j + kApDepth + d < j1 ? j + kApDepth + d : j1 - 1;
            buf[d] = bits[jn * nw + lw];
            if (j + d < j1) {
                // four independent chains: a dependent f64 add would wait for the one before it
                double a4[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int p = 0; p < kApChunkWords; ++p) a4[p & 3] = __builtin_fma(xr[p], ap_sign(ap_word(row, p)), a4[p & 3]);
                double acc = (a4[0] + a4[1]) + (a4[2] + a4[3]);
                acc = ap_wave_sum(acc);
                if (lane == 0) part[chunk * w + j + d] = acc;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Inner pass on the matrix cores (f32 x).  <t_j, x> for many terms j is a dense contraction of a +-1
// matrix with x, so it belongs on MFMA; what keeps it exact is fixed point.  Per chunk of 4096 entries
// x is scaled by a power of two so that |x| 2^s < 2^30, rounded to integers and cut into four balanced
// base-256 digits (int8).  v_mfma_i32_4x4x4_16B_i8 multiplies, in each of its 16 blocks, 4 terms x 4
// entries of signs (int8 +-1, expanded from a nibble of the bitset by a 16-entry table) with 4 entries x
// 4 digits: the four digit columns use the whole instruction, the products and the int32 sums are exact,
// and the digits are recombined in f64.  The only rounding is the fixed point itself: at most
// max|x| 2^-30 per entry of the chunk, below the resolution of the f32 input for all but entries more
// than 64 times smaller than the largest.
// Operand layout of the instruction (lane l, block l / 4): A = row (l % 4) of the block's 4 x 4 sign
// matrix (4 bytes along the contraction), B = column (l % 4) of its 4 x 4 digit matrix (4 bytes along the
// contraction), D register r = element (row r, column l % 4).  Lane = term, so A comes from the lane's
// own row of sign bits; the digit matrix is the same for every block.
typedef int ap_int4 __attribute__((ext_vector_type(4)));

constexpr int kApMfmaWaves = 8;                      // waves per workgroup: each takes 8 of the chunk's 64 words
constexpr int kApTileWords = kApChunkWords / kApMfmaWaves;  // words of a row per wave (64 bytes per term)
constexpr int kApTilePitch = kApTileWords + 1;       // LDS pitch in words: rows 72 bytes apart
static_assert(kApTileWords == 8, "staging below assumes 8 words per wave");

// part[chunk * w + j] = <t_j, x> restricted to the chunk: each wave forms the sum over its 512 entries, the
// eight are joined in wave order through LDS
__global__ void __launch_bounds__(kApMfmaWaves* kWave)
    apply_inner_mfma_kernel(const uint64_t* __restrict__ bits, int64_t nw, int64_t w, const float* __restrict__ x, int64_t n,
                            double* __restrict__ part, int tiles_per_wg)
{
    __shared__ int xd[kApChunkWords * 16 * 4];                    // [group of 4 entries][digit]: 4 packed int8
    __shared__ int lut[16];                                       // nibble -> 4 packed int8 signs
    __shared__ uint64_t tile[kApMfmaWaves][kWave * kApTilePitch];  // per wave: 64 terms x 8 words
    __shared__ float redmax[kApMfmaWaves];
    __shared__ double wsum[kApMfmaWaves][kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int64_t chunk = blockIdx.y;
    const int64_t p0 = chunk * kApChunkWords;
    const int nwc = (int)(nw - p0 < kApChunkWords ? nw - p0 : kApChunkWords);

    // the first tile of sign bits is requested before anything else: its latency hides behind the fixed point
    const int pw = wv * kApTileWords;  // first word of this wave within the chunk
    uint64_t stage[8];
    auto fetch = [&](int64_t jbase) {
        // lane l fetches word (l % 8) of terms (l / 8) + 8 r: every load reads 8 rows x 64 bytes
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            int64_t j = jbase + (lane >> 3) + 8 * r;
            j = j < w ? j : w - 1;
            int p = pw + (lane & 7);
            p = p < nwc ? p : nwc - 1;
            stage[r] = bits[j * nw + p0 + p];
        }
    };
    fetch((int64_t)blockIdx.x * tiles_per_wg * kWave);

    // ---- fixed point of this chunk of x: thread t owns the groups of four entries t and t + 512
    float xv[2][4];
    float amax = 0.f;
    bool finite = true;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int64_t l = p0 * 64 + 4 * (tid + 512 * r) + k;
            const float v = x[l < n ? l : n - 1];
            xv[r][k] = l < n ? v : 0.f;
            finite = finite && (fabsf(xv[r][k]) <= 3.0e38f);
            amax = fmaxf(amax, fabsf(xv[r][k]));
        }
    amax = ap_wave_max(amax);
    if (tid < 16) {
        uint32_t v = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) v |= (((tid >> k) & 1) ? 0xFFu : 0x01u) << (8 * k);
        lut[tid] = (int)v;
    }
    if (lane == 0) redmax[wv] = amax;
    const bool all_finite = !__syncthreads_or(finite ? 0 : 1);
    amax = 0.f;
#pragma unroll
    for (int q = 0; q < kApMfmaWaves; ++q) amax = fmaxf(amax, redmax[q]);
    int ex = 0;
    if (amax > 0.f) (void)frexpf(amax, &ex);  // amax < 2^ex
    const int sh = 30 - ex;
    const double scale = ldexp(1.0, sh), inv_scale = ldexp(1.0, -sh);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        uint32_t dig[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int q = all_finite ? (int)rint((double)xv[r][k] * scale) : 0;
#pragma unroll
            for (int jd = 0; jd < 3; ++jd) {
                const int d = (int)(int8_t)(q & 0xFF);
                dig[jd] |= (uint32_t)(d & 0xFF) << (8 * k);
                q = (q - d) >> 8;
            }
            dig[3] |= (uint32_t)(q & 0xFF) << (8 * k);
        }
        const int g = tid + 512 * r;
#pragma unroll
        for (int jd = 0; jd < 4; ++jd) xd[g * 4 + jd] = (int)dig[jd];
    }
    __syncthreads();

    uint64_t* mytile = tile[wv];
    const int jd = lane & 3;
    const double digit_weight = (double)(1u << (8 * jd));
    double* mypart = part + chunk * w;
    for (int t = 0; t < tiles_per_wg; ++t) {
        const int64_t jbase = ((int64_t)blockIdx.x * tiles_per_wg + t) * kWave;
        if (jbase >= w) break;
        ap_int4 acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
        if (pw < nwc) {
#pragma unroll
            for (int r = 0; r < 8; ++r) mytile[((lane >> 3) + 8 * r) * kApTilePitch + (lane & 7)] = stage[r];
            if (t + 1 < tiles_per_wg && jbase + kWave < w) fetch(jbase + kWave);  // the next 64 terms, during the products
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int pp = 0; pp < kApTileWords; ++pp) {
                if (pw + pp < nwc) {
                    const uint64_t word = mytile[lane * kApTilePitch + pp];
                    const uint32_t half[2] = {(uint32_t)word, (uint32_t)(word >> 32)};
                    const int* xg = xd + ((pw + pp) * 16) * 4 + jd;
#pragma unroll
                    for (int q = 0; q < 16; ++q) {
                        const uint32_t hw = half[q >> 3];
                        const int s4 = 4 * (q & 7);
                        const uint32_t off = s4 >= 2 ? ((hw >> (s4 - 2)) & 0x3Cu) : ((hw << 2) & 0x3Cu);
                        const int a = *(const int*)((const char*)lut + off);
                        if (q & 1) acc1 = __builtin_amdgcn_mfma_i32_4x4x4i8(a, xg[q * 4], acc1, 0, 0, 0);
                        else acc0 = __builtin_amdgcn_mfma_i32_4x4x4i8(a, xg[q * 4], acc0, 0, 0, 0);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();  // the tile is rewritten for the next 64 terms
        }
        // D register i = term jbase + 4 (lane / 4) + i, digit (lane % 4): recombine the digits (exact in f64)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            double v = (double)(acc0[i] + acc1[i]) * digit_weight;
            v += ap_dpp_xor_f64<1>(v);
            v += ap_dpp_xor_f64<2>(v);
            if (jd == 0) wsum[wv][4 * (lane >> 2) + i] = v;
        }
        __syncthreads();  // (every wave of the workgroup runs the same tiles)
        if (wv == 0) {
            double tot = 0.0;
#pragma unroll
            for (int q = 0; q < kApMfmaWaves; ++q) tot += wsum[q][lane];
            const int64_t j = jbase + lane;
            if (j < w) mypart[j] = all_finite ? tot * inv_scale : __longlong_as_double(0x7FF8000000000000ll);
        }
        __syncthreads();  // wsum is rewritten for the next tile
    }
}

// sum over the chunks of <t_j, x>, in order; four loads in flight at a time (a loop that adds each part before
// it loads the next would pay a trip to memory per chunk)
__device__ __forceinline__ double ap_sum_parts(const double* __restrict__ part, int64_t w, int64_t jc, int chunks)
{
    double s = 0.0;
    for (int q0 = 0; q0 < chunks; q0 += 4) {
        double v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = q0 + u < chunks ? part[(int64_t)(q0 + u) * w + jc] : 0.0;
#pragma unroll
        for (int u = 0; u < 4; ++u) s += v[u];
    }
    return s;
}

// Outer pass.  Wave (p, split) owns the 64 output entries of word p and the terms of its split; lane q
// fetches word p of term (tile + q) and forms z of that term (the scale step: c times the chunk parts in
// order); z goes through a wave-private strip of LDS so that every lane can read every term's value.
template <typename TE>
__global__ void __launch_bounds__(kApOuterWaves* kWave)
    apply_outer_kernel(const uint64_t* __restrict__ bits, int64_t mw, int64_t w, const double* __restrict__ part, int chunks,
                       const TE* __restrict__ c, int64_t terms_per_split, double* __restrict__ ypart)
{
    __shared__ double zs[kApOuterWaves][2][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t p = (int64_t)blockIdx.x * kApOuterWaves + wv;  // word of the output this wave owns
    if (p >= mw) return;                                           // (no workgroup-wide barrier below)
    const int64_t split = blockIdx.y;
    const int64_t j0 = split * terms_per_split;
    const int64_t j1 = j0 + terms_per_split < w ? j0 + terms_per_split : w;
    auto fetch = [&](int64_t tile, uint64_t& word, double& z) {
        // unconditional loads; terms past the end re-read the last one and count as z = 0
        const int64_t j = tile + lane;
        const int64_t jc = j < j1 ? j : j1 - 1;
        word = bits[jc * mw + p];
        const double s = ap_sum_parts(part, w, jc, chunks);
        z = j < j1 ? (double)c[jc] * s : 0.0;
    };
    double a4[4] = {0.0, 0.0, 0.0, 0.0};
    if (j0 < j1) {
        // two tiles of 64 terms in flight ahead of the one being added
        uint64_t word_a, word_b;
        double z_a, z_b;
        fetch(j0, word_a, z_a);
        fetch(j0 + kWave < j1 ? j0 + kWave : j0, word_b, z_b);
        int b = 0;
        for (int64_t tile = j0; tile < j1; tile += kWave, b ^= 1) {
            const uint64_t word = word_a;
            zs[wv][b][lane] = z_a;
            word_a = word_b;
            z_a = z_b;
            fetch(tile + 2 * kWave < j1 ? tile + 2 * kWave : tile, word_b, z_b);
            // the strip is written and read by this wave only: LDS operations of one wave complete in order
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll 16
            for (int q = 0; q < kWave; ++q) a4[q & 3] = __builtin_fma(zs[wv][b][q], ap_sign(ap_word(word, q)), a4[q & 3]);
        }
    }
    ypart[split * (mw * 64) + p * 64 + lane] = (a4[0] + a4[1]) + (a4[2] + a4[3]);
}

// ------------------------------------------------------------------------------------------------
// Outer pass on the matrix cores (f32).  y_i = sum_j z_j s_j[i] is the same kind of contraction as the
// inner pass with the roles swapped: the terms are the contraction index and z plays the part of x (block
// fixed point per split of the terms: |z| 2^s < 2^30, four balanced base-256 digits, at most
// max|z| 2^-30 per term, exact sums afterwards).  The bitset is term-major, so the four signs an
// instruction wants per lane (one output entry, four consecutive terms) sit in four different words:
// a wave loads word p of 64 consecutive terms (one per lane) and transposes the 64 x 64 bits across
// its lanes (six butterfly stages); lane i then holds the signs of output entry 64 p + i for the 64 terms,
// packed along the contraction exactly as the inner pass has them.
constexpr int kApFxMaxTerms = 2048;  // terms per split: one group of four per thread of the workgroup
// digits of one kind are kApFxPitch words apart: the four that a wave reads together fall into different banks
constexpr int kApFxPitch = kApFxMaxTerms / 4 + 4;

// 64 x 64 bit transpose across a wave: lane q brings row q (bit i = column i), lane i leaves with column i.
// Six butterfly stages (distance 32, 16, .., 1): in every 2s x 2s block the two off-diagonal s x s blocks
// change places, the partner row is s lanes away.  The rows are kept as two 32-bit halves; below distance
// 32 a stage is, per half, one lane exchange, one rotate (the partner's bits move s columns up in the
// upper row, s down in the lower) and one bitfield insert.  Distances 1..8 stay within a row of 16 lanes
// and use the data-parallel lane modes, distances 16 and 32 the row-swap instructions (no LDS traffic).
template <int S>
__device__ __forceinline__ uint32_t ap_lane_xor(uint32_t v, int lane)
{
    if constexpr (S == 1) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0xB1, 0xF, 0xF, true);  // quad_perm 1,0,3,2
    else if constexpr (S == 2) return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, 0x4E, 0xF, 0xF, true);  // quad_perm 2,3,0,1
    else if constexpr (S == 4) {
        // lane ^ 7 (mirror of half a row), then lane ^ 3 (quad_perm 3,2,1,0)
        const int h = __builtin_amdgcn_mov_dpp((int)v, 0x141, 0xF, 0xF, true);
        return (uint32_t)__builtin_amdgcn_mov_dpp(h, 0x1B, 0xF, 0xF, true);
    } else if constexpr (S == 8) {
        // lane ^ 15 (mirror of a row), then lane ^ 7
        const int h = __builtin_amdgcn_mov_dpp((int)v, 0x140, 0xF, 0xF, true);
        return (uint32_t)__builtin_amdgcn_mov_dpp(h, 0x141, 0xF, 0xF, true);
    } else {
        // distance 16 or 32: the row swap leaves (value of the lower partner, value of the upper partner) in
        // both lanes; each takes the other's
        uint32_t a, b;
        ap_swap_pair<S>(v, a, b);
        return (lane & S) ? a : b;
    }
}

template <int S>
__device__ __forceinline__ uint32_t ap_butterfly(uint32_t h, int lane)
{
    constexpr uint32_t m = S == 16 ? 0x0000FFFFu : S == 8 ? 0x00FF00FFu : S == 4 ? 0x0F0F0F0Fu : S == 2 ? 0x33333333u : 0x55555555u;
    const bool lower = (lane & S) != 0;
    const uint32_t p = ap_lane_xor<S>(h, lane);
    const uint32_t rot = __builtin_amdgcn_alignbit(p, p, lower ? S : 32 - S);  // partner >> S (lower row), << S (upper)
    const uint32_t keep = lower ? ~m : m;
    return (h & keep) | (rot & ~keep);
}

__device__ __forceinline__ uint64_t ap_transpose64(uint64_t x, int lane)
{
    uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
    {
        // distance 32: the upper rows take the partner's low half as their high half, the lower rows the
        // partner's high half as their low half
        const bool lower = (lane & 32) != 0;
        const uint32_t got = ap_lane_xor<32>(lower ? lo : hi, lane);
        lo = lower ? got : lo;
        hi = lower ? hi : got;
    }
    lo = ap_butterfly<16>(lo, lane), hi = ap_butterfly<16>(hi, lane);
    lo = ap_butterfly<8>(lo, lane), hi = ap_butterfly<8>(hi, lane);
    lo = ap_butterfly<4>(lo, lane), hi = ap_butterfly<4>(hi, lane);
    lo = ap_butterfly<2>(lo, lane), hi = ap_butterfly<2>(hi, lane);
    lo = ap_butterfly<1>(lo, lane), hi = ap_butterfly<1>(hi, lane);
    return ((uint64_t)hi << 32) | lo;
}

__global__ void __launch_bounds__(kApMfmaWaves* kWave)
    apply_outer_mfma_kernel(const uint64_t* __restrict__ bits, int64_t mw, int64_t w, const double* __restrict__ part,
                            int chunks, const float* __restrict__ c, int64_t terms_per_split, double* __restrict__ ypart)
{
    __shared__ __align__(16) int zd[4 * kApFxPitch];  // [digit][group of 4 terms]: 4 packed int8
    __shared__ int lut[16];            // nibble -> 4 packed int8 signs
    __shared__ double redmax[kApMfmaWaves];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int64_t p = (int64_t)blockIdx.x * kApMfmaWaves + wv;  // word of the output this wave owns
    const int64_t pc = p < mw ? p : mw - 1;
    const int64_t split = blockIdx.y;
    const int64_t j0 = split * terms_per_split;
    const int64_t j1 = j0 + terms_per_split < w ? j0 + terms_per_split : w;  // (the plan leaves no split empty)
    // lane q fetches word p of term (tile + q); terms past the end re-read the last one (their z is zero)
    auto fetch = [&](int64_t tile) {
        const int64_t j = j0 + tile * kWave + lane;
        return bits[(j < j1 ? j : j1 - 1) * mw + pc];
    };
    uint64_t next = fetch(0);

    // ---- z of this split in fixed point: thread t owns the group of four terms t
    double zv[4];
    double amax = 0.0;
    bool finite = true;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int64_t j = j0 + 4 * tid + k;
        const int64_t jc = j < j1 ? j : j1 - 1;
        const double s = ap_sum_parts(part, w, jc, chunks);
        zv[k] = j < j1 ? (double)c[jc] * s : 0.0;
        finite = finite && (fabs(zv[k]) <= 1.7e308);
        amax = fmax(amax, fabs(zv[k]));
    }
    amax = ap_wave_max(amax);
    if (tid < 16) {
        uint32_t v = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) v |= (((tid >> k) & 1) ? 0xFFu : 0x01u) << (8 * k);
        lut[tid] = (int)v;
    }
    if (lane == 0) redmax[wv] = amax;
    const bool all_finite = !__syncthreads_or(finite ? 0 : 1);
    amax = 0.0;
#pragma unroll
    for (int q = 0; q < kApMfmaWaves; ++q) amax = fmax(amax, redmax[q]);
    int ex = 0;
    if (amax > 0.0) (void)frexp(amax, &ex);  // amax < 2^ex
    int sh = 30 - ex;
    sh = sh > 1000 ? 1000 : sh;              // (2^sh stays a normal number; smaller z round to zero)
    const double scale = ldexp(1.0, sh), inv_scale = ldexp(1.0, -sh);
    {
        uint32_t dig[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int q = all_finite ? (int)rint(zv[k] * scale) : 0;
#pragma unroll
            for (int jd = 0; jd < 3; ++jd) {
                const int d = (int)(int8_t)(q & 0xFF);
                dig[jd] |= (uint32_t)(d & 0xFF) << (8 * k);
                q = (q - d) >> 8;
            }
            dig[3] |= (uint32_t)(q & 0xFF) << (8 * k);
        }
#pragma unroll
        for (int jd = 0; jd < 4; ++jd) zd[jd * kApFxPitch + tid] = (int)dig[jd];
    }
    __syncthreads();
    if (p >= mw) return;  // (no workgroup-wide barrier below)

    const int jd = lane & 3;
    const int ntiles = (int)((j1 - j0 + kWave - 1) / kWave);
    ap_int4 acc0 = {0, 0, 0, 0}, acc1 = {0, 0, 0, 0};
    for (int t = 0; t < ntiles; ++t) {
        const uint64_t mine = next;
        if (t + 1 < ntiles) next = fetch(t + 1);
        const uint64_t col = ap_transpose64(mine, lane);  // bit q: sign of term (tile + q) at this lane's entry
        const uint32_t half[2] = {(uint32_t)col, (uint32_t)(col >> 32)};
        // this lane's digit of the tile's 16 groups of four terms (four 16-byte reads)
        const ap_int4* zq = (const ap_int4*)(zd + jd * kApFxPitch + t * 16);
        int zg[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const ap_int4 v = zq[q];
            zg[4 * q] = v[0], zg[4 * q + 1] = v[1], zg[4 * q + 2] = v[2], zg[4 * q + 3] = v[3];
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const uint32_t hw = half[q >> 3];
            const int s4 = 4 * (q & 7);
            const uint32_t off = s4 >= 2 ? ((hw >> (s4 - 2)) & 0x3Cu) : ((hw << 2) & 0x3Cu);
            const int a = *(const int*)((const char*)lut + off);
            if (q & 1) acc1 = __builtin_amdgcn_mfma_i32_4x4x4i8(a, zg[q], acc1, 0, 0, 0);
            else acc0 = __builtin_amdgcn_mfma_i32_4x4x4i8(a, zg[q], acc0, 0, 0, 0);
        }
    }
    // D register i = output entry 64 p + 4 (lane / 4) + i, digit (lane % 4): recombine the digits (exact in f64)
    const double digit_weight = (double)(1u << (8 * jd));
    double* out = ypart + split * (mw * 64) + p * 64 + 4 * (lane >> 2);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        double v = (double)(acc0[i] + acc1[i]) * digit_weight;
        v += ap_dpp_xor_f64<1>(v);
        v += ap_dpp_xor_f64<2>(v);
        if (jd == 0) out[i] = all_finite ? v * inv_scale : __longlong_as_double(0x7FF8000000000000ll);
    }
}

// y = sum of the splits in order, rounded once.  64 entries per workgroup; the splits are cut into four
// runs that are added side by side (their loads in flight together) and joined in order.
template <typename TE>
__global__ void __launch_bounds__(256)
    apply_reduce_kernel(const double* __restrict__ ypart, int splits, int64_t mpad, int64_t m, TE* __restrict__ y)
{
    __shared__ double run[4][64];
    const int r = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + r;
    const int per = (splits + 3) / 4;
    const int q0 = g * per, q1 = q0 + per < splits ? q0 + per : splits;
    double s = 0.0;
    if (i < mpad) {
        int q = q0;
        for (; q + 4 <= q1; q += 4) {
            const double a0 = ypart[(int64_t)q * mpad + i], a1 = ypart[(int64_t)(q + 1) * mpad + i];
            const double a2 = ypart[(int64_t)(q + 2) * mpad + i], a3 = ypart[(int64_t)(q + 3) * mpad + i];
            s = (((s + a0) + a1) + a2) + a3;
        }
        for (; q < q1; ++q) s += ypart[(int64_t)q * mpad + i];
    }
    run[g][r] = s;
    __syncthreads();
    if (g == 0 && i < m) y[i] = (TE)(((run[0][r] + run[1][r]) + run[2][r]) + run[3][r]);
}

}  // namespace

void apply_plan(int64_t nin, int64_t nout, int64_t w, ApplyPlan* pl)
{
    const int64_t win = (nin + 63) / 64, wout = (nout + 63) / 64;
    pl->chunks = (int)((win + kApChunkWords - 1) / kApChunkWords);
    if (pl->chunks < 1) pl->chunks = 1;
    // inner pass: enough waves to fill the device, enough terms per wave to pay for loading its chunk of x
    int64_t tpw = (w * pl->chunks + 4095) / 4096;
    if (tpw < 8) tpw = 8;
    if (tpw > 64) tpw = 64;
    pl->terms_per_wave = (int)tpw;
    // outer pass: one wave per word of the output and split of the terms
    int64_t splits = wout > 0 ? (4096 + wout - 1) / wout : 1;
    if (splits > 64) splits = 64;
    while (splits > 1 && (w + splits - 1) / splits < 32) --splits;
    if (splits < 1) splits = 1;
    pl->terms_per_split = (w + splits - 1) / splits;
    if (pl->terms_per_split < 1) pl->terms_per_split = 1;
    pl->splits = (int)((w + pl->terms_per_split - 1) / pl->terms_per_split);
    if (pl->splits < 1) pl->splits = 1;
    // outer pass in fixed point (f32): a workgroup takes 8 words of the output and one split of the terms
    // (whole tiles of 64, at most kApFxMaxTerms); two to four workgroups per compute unit
    {
        const int64_t gx = (wout + kApMfmaWaves - 1) / kApMfmaWaves;
        const int64_t target = gx >= 16 ? 1024 : 512;
        int64_t want = gx > 0 ? (target + gx - 1) / gx : 1;
        const int64_t least = (w + kApFxMaxTerms - 1) / kApFxMaxTerms, most = (w + kWave - 1) / kWave;
        if (want > most) want = most;
        if (want < least) want = least;
        if (want < 1) want = 1;
        int64_t tps = ((w + want - 1) / want + kWave - 1) / kWave * kWave;
        if (tps < kWave) tps = kWave;
        pl->terms_per_split_fx = tps;
        pl->splits_fx = (int)((w + tps - 1) / tps);
        if (pl->splits_fx < 1) pl->splits_fx = 1;
    }
    pl->off_part = 0;
    pl->parts = pl->chunks;  // slices of <t_j, x> the inner pass writes per term
    pl->off_ypart = pl->off_part + (size_t)pl->parts * (size_t)w * 8;
    const int most_splits = pl->splits > pl->splits_fx ? pl->splits : pl->splits_fx;
    pl->bytes = pl->off_ypart + (size_t)most_splits * (size_t)wout * 64 * 8;
    if (pl->bytes < 8) pl->bytes = 8;
}

hipError_t launch_apply(const uint64_t* in_bits, const uint64_t* out_bits, const void* c, scd_dtype dt, int64_t nin,
                        int64_t nout, int64_t w, const void* x, void* y, void* workspace, hipStream_t st)
{
    ApplyPlan pl;
    apply_plan(nin, nout, w, &pl);
    const int64_t win = (nin + 63) / 64, wout = (nout + 63) / 64;
    double* part = (double*)((char*)workspace + pl.off_part);
    double* ypart = (double*)((char*)workspace + pl.off_ypart);
    if (nout == 0) return hipSuccess;
    if (w == 0 || nin == 0) {
        // the empty sum: a reduce over no splits writes zeros
        const unsigned g0 = (unsigned)((nout + 63) / 64);
        if (dt == SCD_F32)
            hipLaunchKernelGGL((apply_reduce_kernel<float>), dim3(g0), dim3(256), 0, st, ypart, 0, wout * 64, nout, (float*)y);
        else
            hipLaunchKernelGGL((apply_reduce_kernel<double>), dim3(g0), dim3(256), 0, st, ypart, 0, wout * 64, nout, (double*)y);
        return hipGetLastError();
    }
    const int64_t waves = (w + pl.terms_per_wave - 1) / pl.terms_per_wave;
    dim3 gi((unsigned)((waves + kApInnerWaves - 1) / kApInnerWaves), (unsigned)pl.chunks);
    if (dt == SCD_F32) {
        // one workgroup per tile of 64 terms (eight waves split the chunk's words); several tiles per
        // workgroup once there are enough of them, to pay for the fixed point less often
        const int64_t tiles = (w + kWave - 1) / kWave;
        int tpw = (int)((tiles * pl.chunks + 1023) / 1024);
        if (tpw < 1) tpw = 1;
        const int64_t wgs = (tiles + tpw - 1) / tpw;
        hipLaunchKernelGGL(apply_inner_mfma_kernel, dim3((unsigned)wgs, (unsigned)pl.chunks), dim3(kApMfmaWaves * kWave), 0, st,
                           in_bits, win, w, (const float*)x, nin, part, tpw);
    } else
        hipLaunchKernelGGL((apply_inner_kernel<double>), gi, dim3(kApInnerWaves * kWave), 0, st, in_bits, win, w,
                           (const double*)x, nin, part, pl.terms_per_wave);
    dim3 go((unsigned)((wout + kApOuterWaves - 1) / kApOuterWaves), (unsigned)pl.splits);
    if (dt == SCD_F32) {
        dim3 gf((unsigned)((wout + kApMfmaWaves - 1) / kApMfmaWaves), (unsigned)pl.splits_fx);
        hipLaunchKernelGGL(apply_outer_mfma_kernel, gf, dim3(kApMfmaWaves * kWave), 0, st, out_bits, wout, w, part, pl.parts,
                           (const float*)c, pl.terms_per_split_fx, ypart);
    } else
        hipLaunchKernelGGL((apply_outer_kernel<double>), go, dim3(kApOuterWaves * kWave), 0, st, out_bits, wout, w, part,
                           pl.parts, (const double*)c, pl.terms_per_split, ypart);
    const unsigned gr = (unsigned)((nout + 63) / 64);
    if (dt == SCD_F32)
        hipLaunchKernelGGL((apply_reduce_kernel<float>), dim3(gr), dim3(256), 0, st, ypart, pl.splits_fx, wout * 64, nout, (float*)y);
    else
        hipLaunchKernelGGL((apply_reduce_kernel<double>), dim3(gr), dim3(256), 0, st, ypart, pl.splits, wout * 64, nout, (double*)y);
    return hipGetLastError();
}

}  // namespace scd
