// Least squares decomposition (Algorithm 6, Section 3.3 of arXiv 2410.01799): after every greedy signed
// cut the coefficients of ALL terms are refitted, c = argmin ||A - S diag(c) T^T||_F.
//
// The remainder R_k = A - S_k diag(c_k) T_k^T is never formed: every coefficient changes with every term,
// so keeping R up to date would cost a rank-k update per term.  Instead each half step of the cut works on
//     R t   = A t   - S (c o (T^T t)),        R^T s = A^T s - T (c o (S^T s)),
// where A t and A^T s are the ordinary signed-sum passes over A, <t_j, t> = n - 2 popcount(t_j xor t)
// comes from the bitsets, and the correction is a signed sum of k scalars per entry.  The normal equations
// (Section 3.3) use the Gram matrix G_ij = <s_i,s_j><t_i,t_j>, again from popcounts, kept as a Cholesky
// factor that grows by one row per term; b_j = <s_j, A t_j> falls out of the last half step of term j.
// Everything here is f64; the kernels are small and latency-bound (one term = a few hundred launches).
#include "scd_device.h"

namespace scd {

namespace {

__device__ __forceinline__ double lq_wave_sum(double a)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, kWave);
    return a;
}

// out[j] = coef[j] * <x_j, vec> for sign vectors given as bitsets of `len` entries (coef null: 1);
// one wave per term.  Padding bits are zero on both sides.
__global__ void __launch_bounds__(256)
    lsq_dots_kernel(const uint64_t* __restrict__ bits, int64_t k, int64_t nw, int64_t len, const uint64_t* __restrict__ vec,
                    const double* __restrict__ coef, double* __restrict__ out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t j = (int64_t)blockIdx.x * 4 + threadIdx.x / kWave;
    if (j >= k) return;
    int cnt = 0;
    for (int64_t p = lane; p < nw; p += kWave) cnt += __popcll(bits[j * nw + p] ^ vec[p]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, kWave);
    if (lane == 0) {
        const double d = (double)(len - 2 * (int64_t)cnt);
        out[j] = coef ? coef[j] * d : d;
    }
}

// y_i = base_i - sum_{j<k} e_j x_j[i] for the 64 entries of word p = blockIdx.x (lane = entry); the eight
// waves take the terms j = wave, wave + 8, ... and their partial sums are joined in wave order.
// Writes sgn(y) as a word of bits, optionally y, and per word sum |y_i| and sum sgn(y_i) base_i.
__global__ void __launch_bounds__(512)
    lsq_correct_kernel(const uint64_t* __restrict__ bits, int64_t k, int64_t mw, int64_t m, const double* __restrict__ e,
                       const double* __restrict__ base, uint64_t* __restrict__ out_bits, double* __restrict__ abs_parts,
                       double* __restrict__ dot_parts)
{
    __shared__ double part[8][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int64_t p = blockIdx.x;
    double acc = 0.0;
    for (int64_t j = wv; j < k; j += 8) {
        const uint64_t word = bits[j * mw + p];  // the same for all lanes
        const double sgn = __hiloint2double(((word >> lane) & 1ull) ? (int)0xBFF00000 : (int)0x3FF00000, 0);
        acc = __builtin_fma(e[j], sgn, acc);
    }
    part[wv][lane] = acc;
    __syncthreads();
    if (wv != 0) return;
    double tot = 0.0;
#pragma unroll
    for (int q = 0; q < 8; ++q) tot += part[q][lane];
    const int64_t i = p * 64 + lane;
    const bool valid = i < m;
    const double b = valid ? base[i] : 0.0;
    const double y = valid ? b - tot : 0.0;
    const bool neg = y < 0.0;
    const uint64_t bal = __ballot(valid && neg);
    if (lane == 0) out_bits[p] = bal;
    if (abs_parts) {
        const double a = lq_wave_sum(fabs(y));
        const double d = lq_wave_sum(neg ? -b : b);
        if (lane == 0) {
            abs_parts[p] = a;
            dot_parts[p] = d;
        }
    }
}

// out[0] = sum a, out[1] = sum b (b may be null), n values each, in a fixed order (one workgroup)
__global__ void __launch_bounds__(256) lsq_sum2_kernel(const double* __restrict__ a, const double* __restrict__ b, int64_t n,
                                                      double* __restrict__ out)
{
    __shared__ double ra[256], rb[256];
    double sa = 0.0, sb = 0.0;
    for (int64_t i = threadIdx.x; i < n; i += 256) {
        sa += a[i];
        if (b) sb += b[i];
    }
    ra[threadIdx.x] = sa;
    rb[threadIdx.x] = sb;
    __syncthreads();
    if (threadIdx.x == 0) {
        double ta = 0.0, tb = 0.0;
        for (int q = 0; q < 256; ++q) {
            ta += ra[q];
            tb += rb[q];
        }
        out[0] = ta;
        out[1] = tb;
    }
}

template <typename TE>
__global__ void __launch_bounds__(256) lsq_sumsq_kernel(const TE* __restrict__ A, int64_t total, double* __restrict__ parts)
{
    __shared__ double red[256];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const double v = (double)A[i];
        s += v * v;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int q = 0; q < 256; ++q) t += red[q];
        parts[blockIdx.x] = t;
    }
}

template <typename TE>
__global__ void __launch_bounds__(256) lsq_cast_kernel(const double* __restrict__ c, int64_t k, TE* __restrict__ out)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j < k) out[j] = (TE)c[j];
}

// out[j] = (coef ? coef[j] : 1) * product over the modes m != skip of D[m * ld + j]   (skip < 0: all modes)
__global__ void __launch_bounds__(256) lsq_prod_kernel(const double* __restrict__ D, int64_t ld, int order, int skip, int64_t k,
                                                      const double* __restrict__ coef, double* __restrict__ out)
{
    const int64_t j = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= k) return;
    double p = coef ? coef[j] : 1.0;
    for (int m = 0; m < order; ++m)
        if (m != skip) p *= D[(int64_t)m * ld + j];
    out[j] = p;
}

// Sign bits of the tensor product of the sign vectors of modes first..last-1 (last mode fastest): bit q is
// the xor of the modes' bits at the multi-index of q (Algorithm 12 lines 5-7).  One lane per entry.
struct LsqKronArgs {
    const uint64_t* signs[SCD_MAX_ORDER];
    int64_t dims[SCD_MAX_ORDER];
    int first, last;
    int64_t len;
    uint64_t* out;
};

__global__ void __launch_bounds__(256) lsq_kron_kernel(LsqKronArgs a)
{
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    unsigned bit = 0;
    if (q < a.len) {
        int64_t rest = q;
        for (int m = a.last - 1; m >= a.first; --m) {
            const int64_t i = rest % a.dims[m];
            rest /= a.dims[m];
            bit ^= (unsigned)((a.signs[m][i >> 6] >> (i & 63)) & 1ull);
        }
    }
    const uint64_t word = __ballot(q < a.len && bit);
    if ((threadIdx.x & (kWave - 1)) == 0 && (q >> 6) < (a.len + 63) / 64) a.out[q >> 6] = word;
}

// Real last mode: c[ch] = u[ch] / P, rounded to the element type (the stored value is what gets subtracted).
template <typename TE>
__global__ void __launch_bounds__(256) scalars_coef_kernel(const double* __restrict__ u, int64_t q, double P, TE* __restrict__ c)
{
    const int64_t ch = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (ch < q) c[ch] = (TE)(u[ch] / P);
}

// r[p][ch] -= sign_p * c[ch] over the whole tensor (p = index over the leading modes, sign_p = bit p of
// `lead`, a 1 bit standing for -1), and the sum of the squares of what is left, per workgroup.
template <typename TE>
__global__ void __launch_bounds__(256) scalars_update_kernel(TE* __restrict__ r, int64_t total, int64_t q,
                                                            const uint64_t* __restrict__ lead, const TE* __restrict__ c,
                                                            double* __restrict__ parts)
{
    __shared__ double red[256];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t p = i / q, ch = i - p * q;
        const TE d = ((lead[p >> 6] >> (p & 63)) & 1ull) ? -c[ch] : c[ch];
        const TE v = r[i] - d;
        r[i] = v;
        s += (double)v * (double)v;
    }
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = 0.0;
        for (int z = 0; z < 256; ++z) t += red[z];
        parts[blockIdx.x] = t;
    }
}

constexpr int kLqThreads = 1024;

// sum over the workgroup in a fixed order; every thread gets the same bits
__device__ double lq_block_sum(double v, double* red)
{
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    v = lq_wave_sum(v);
    __syncthreads();  // red may still be read from the previous call
    if (lane == 0) red[wv] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < kLqThreads / kWave; ++q) t += red[q];
    return t;
}

// The new term has index k.  Appends row k to the Cholesky factor L (lower triangular, row-major, leading
// dimension ld) of the Gram matrix, whose new row is g[j] (j < k) with `diag` on the diagonal;
// extends the forward solution y of L y = b by one entry; solves L^T c = y for all k + 1 coefficients;
// and records ||A - S diag(c) T^T||_F = sqrt(||A||^2 - <c, b>) (the remainder is orthogonal to the fit).
// One workgroup.  status: 1 if the new term is (numerically) in the span of the old ones.
__global__ void __launch_bounds__(kLqThreads)
    lsq_solve_kernel(double* __restrict__ L, int64_t ld, int64_t k, const double* __restrict__ g, double diag, const double* __restrict__ bvec, double* __restrict__ yv, double* __restrict__ c,
                     double* __restrict__ work, double fro0sq, double* __restrict__ trace_out, int* __restrict__ status)
{
    __shared__ double red[kLqThreads / kWave];
    const int tid = threadIdx.x;
    double* row = L + k * ld;
    // ---- forward substitution: row_r = (g_r - sum_{q<r} L[r][q] row_q) / L[r][r]
    for (int64_t r = 0; r < k; ++r) {
        double s = 0.0;
        for (int64_t q = tid; q < r; q += kLqThreads) s += L[r * ld + q] * row[q];
        s = lq_block_sum(s, red);
        if (tid == 0) row[r] = (g[r] - s) / L[r * ld + r];
        __threadfence_block();
        __syncthreads();
    }
    double s2 = 0.0, sy = 0.0;
    for (int64_t q = tid; q < k; q += kLqThreads) {
        s2 += row[q] * row[q];
        sy += row[q] * yv[q];
    }
    s2 = lq_block_sum(s2, red);
    sy = lq_block_sum(sy, red);
    const double d2 = diag - s2;
    if (!(d2 > 1e-9 * diag)) {
        if (tid == 0) *status = 1;
        return;
    }
    const double lkk = sqrt(d2);
    if (tid == 0) {
        row[k] = lkk;
        yv[k] = (bvec[k] - sy) / lkk;
    }
    __threadfence_block();
    __syncthreads();
    // ---- back substitution L^T c = y, in axpy form: rows of L are contiguous
    for (int64_t q = tid; q <= k; q += kLqThreads) work[q] = yv[q];
    __threadfence_block();
    __syncthreads();
    for (int64_t r = k; r >= 0; --r) {
        const double cr = work[r] / L[r * ld + r];
        if (tid == 0) c[r] = cr;
        for (int64_t q = tid; q < r; q += kLqThreads) work[q] -= L[r * ld + q] * cr;
        __threadfence_block();
        __syncthreads();
    }
    double cb = 0.0;
    for (int64_t q = tid; q <= k; q += kLqThreads) cb += c[q] * bvec[q];
    cb = lq_block_sum(cb, red);
    if (tid == 0) {
        const double f2 = fro0sq - cb;
        trace_out[0] = sqrt(f2 > 0.0 ? f2 : 0.0);
    }
}

}  // namespace

hipError_t launch_lsq_dots(const uint64_t* bits, int64_t k, int64_t nw, int64_t len, const uint64_t* vec, const double* coef,
                           double* out, hipStream_t st)
{
    if (k <= 0) return hipSuccess;
    hipLaunchKernelGGL(lsq_dots_kernel, dim3((unsigned)((k + 3) / 4)), dim3(256), 0, st, bits, k, nw, len, vec, coef, out);
    return hipGetLastError();
}

hipError_t launch_lsq_correct(const uint64_t* bits, int64_t k, int64_t mw, int64_t m, const double* e, const double* base,
                              uint64_t* out_bits, double* abs_parts, double* dot_parts, hipStream_t st)
{
    hipLaunchKernelGGL(lsq_correct_kernel, dim3((unsigned)mw), dim3(512), 0, st, bits, k, mw, m, e, base, out_bits, abs_parts,
                       dot_parts);
    return hipGetLastError();
}

hipError_t launch_lsq_prod(const double* D, int64_t ld, int order, int skip, int64_t k, const double* coef, double* out,
                           hipStream_t st)
{
    if (k <= 0) return hipSuccess;
    hipLaunchKernelGGL(lsq_prod_kernel, dim3((unsigned)((k + 255) / 256)), dim3(256), 0, st, D, ld, order, skip, k, coef, out);
    return hipGetLastError();
}

hipError_t launch_lsq_kron(const uint64_t* const* signs, const int64_t* dims, int first, int last, int64_t len, uint64_t* out,
                           hipStream_t st)
{
    LsqKronArgs a;
    for (int m = 0; m < SCD_MAX_ORDER; ++m) {
        a.signs[m] = (m >= first && m < last) ? signs[m] : nullptr;
        a.dims[m] = (m >= first && m < last) ? dims[m] : 1;
    }
    a.first = first;
    a.last = last;
    a.len = len;
    a.out = out;
    const int64_t padded = ((len + 63) / 64) * 64;
    hipLaunchKernelGGL(lsq_kron_kernel, dim3((unsigned)((padded + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_scalars_coef(const double* u, int64_t q, double P, scd_dtype dt, void* c, hipStream_t st)
{
    const unsigned g = (unsigned)((q + 255) / 256);
    if (dt == SCD_F32)
        hipLaunchKernelGGL((scalars_coef_kernel<float>), dim3(g), dim3(256), 0, st, u, q, P, (float*)c);
    else
        hipLaunchKernelGGL((scalars_coef_kernel<double>), dim3(g), dim3(256), 0, st, u, q, P, (double*)c);
    return hipGetLastError();
}

hipError_t launch_scalars_update(void* r, scd_dtype dt, int64_t total, int64_t q, const uint64_t* lead, const void* c,
                                 double* parts, int nparts, hipStream_t st)
{
    if (dt == SCD_F32)
        hipLaunchKernelGGL((scalars_update_kernel<float>), dim3(nparts), dim3(256), 0, st, (float*)r, total, q, lead,
                           (const float*)c, parts);
    else
        hipLaunchKernelGGL((scalars_update_kernel<double>), dim3(nparts), dim3(256), 0, st, (double*)r, total, q, lead,
                           (const double*)c, parts);
    return hipGetLastError();
}

hipError_t launch_lsq_sum2(const double* a, const double* b, int64_t n, double* out, hipStream_t st)
{
    hipLaunchKernelGGL(lsq_sum2_kernel, dim3(1), dim3(256), 0, st, a, b, n, out);
    return hipGetLastError();
}

hipError_t launch_lsq_sumsq(const void* A, scd_dtype dt, int64_t total, double* parts, int nparts, hipStream_t st)
{
    if (dt == SCD_F32)
        hipLaunchKernelGGL((lsq_sumsq_kernel<float>), dim3(nparts), dim3(256), 0, st, (const float*)A, total, parts);
    else
        hipLaunchKernelGGL((lsq_sumsq_kernel<double>), dim3(nparts), dim3(256), 0, st, (const double*)A, total, parts);
    return hipGetLastError();
}

hipError_t launch_lsq_cast(const double* c, int64_t k, scd_dtype dt, void* out, hipStream_t st)
{
    if (k <= 0) return hipSuccess;
    const unsigned g = (unsigned)((k + 255) / 256);
    if (dt == SCD_F32)
        hipLaunchKernelGGL((lsq_cast_kernel<float>), dim3(g), dim3(256), 0, st, c, k, (float*)out);
    else
        hipLaunchKernelGGL((lsq_cast_kernel<double>), dim3(g), dim3(256), 0, st, c, k, (double*)out);
    return hipGetLastError();
}

hipError_t launch_lsq_solve(double* L, int64_t ld, int64_t k, const double* g, double diag, const double* bvec, double* yv,
                            double* c, double* work, double fro0sq, double* trace_out, int* status, hipStream_t st)
{
    hipLaunchKernelGGL(lsq_solve_kernel, dim3(1), dim3(kLqThreads), 0, st, L, ld, k, g, diag, bvec, yv, c, work, fro0sq,
                       trace_out, status);
    return hipGetLastError();
}

}  // namespace scd
