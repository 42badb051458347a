/* Drives every entry point of the CPU oracle on small ragged inputs; built by tests/test_oracle_sanitizers.py
 * together with oracle/scd_oracle.c under -fsanitize=address,undefined.  Exit code 0 and silence = clean. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int scdo_decompose(const double*, int64_t, int64_t, int64_t, uint64_t, int32_t, uint64_t*, uint64_t*, double*, double*,
                   int32_t*, double*, double*);
int scdo_lsq_decompose(const double*, int64_t, int64_t, int64_t, uint64_t, int32_t, uint64_t*, uint64_t*, double*, double*,
                       int32_t*, double*);
int scdo_tensor_decompose(const double*, int, const int64_t*, int64_t, uint64_t, int32_t, uint64_t* const*, double*, double*,
                          int32_t*, double*, double*);
int scdo_tensor_lsq_decompose(const double*, int, const int64_t*, int64_t, uint64_t, int32_t, uint64_t* const*, double*,
                              double*, int32_t*, double*);
int scdo_scalars_decompose(const double*, int, const int64_t*, int64_t, uint64_t, int32_t, uint64_t* const*, double*, double*,
                           int32_t*, double*);
void scdo_expand(int, const int64_t*, int64_t, const uint64_t* const*, const double*, double*);
void scdo_apply(int64_t, int64_t, int64_t, const uint64_t*, const uint64_t*, const double*, int, const double*, double*);
double scdo_bruteforce_signed_cut_norm(const double*, int64_t, int64_t, uint64_t*);

static double noise(uint64_t* state)
{
    *state = *state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)((*state >> 11) & 0xFFFFF) / 524288.0 - 1.0;
}

int main(void)
{
    const int64_t shapes[][2] = {{1, 1}, {7, 130}, {65, 64}, {33, 5}};
    uint64_t st = 7;
    for (unsigned q = 0; q < sizeof(shapes) / sizeof(shapes[0]); ++q) {
        const int64_t m = shapes[q][0], n = shapes[q][1], w = 5;
        const int64_t mw = (m + 63) / 64, nw = (n + 63) / 64;
        double* A = malloc(sizeof(double) * m * n);
        for (int64_t i = 0; i < m * n; ++i) A[i] = noise(&st);
        uint64_t* S = calloc(w * mw, 8);
        uint64_t* T = calloc(w * nw, 8);
        double c[5], trace[6], margins[10];
        int32_t iters[5];
        double* R = malloc(sizeof(double) * m * n);
        scdo_decompose(A, m, n, w, 3, 64, S, T, c, trace, iters, margins, R);
        if (!(trace[w] <= trace[0])) return 2;
        const int64_t dims[2] = {m, n};
        const uint64_t* sg[2] = {S, T};
        double* E = malloc(sizeof(double) * m * n);
        scdo_expand(2, dims, w, sg, c, E);
        double* x = malloc(sizeof(double) * (m > n ? m : n));
        double* y = malloc(sizeof(double) * (m > n ? m : n));
        for (int64_t i = 0; i < (m > n ? m : n); ++i) x[i] = noise(&st);
        scdo_apply(m, n, w, S, T, c, 0, x, y);
        scdo_apply(m, n, w, S, T, c, 1, x, y);
        if (m * n > 4 && scdo_lsq_decompose(A, m, n, 3, 3, 64, S, T, c, trace, iters, margins) < 0) return 3;
        if (m <= 8) {
            uint64_t best;
            if (!(scdo_bruteforce_signed_cut_norm(A, m, n, &best) >= 0.0)) return 4;
        }
        free(A); free(S); free(T); free(R); free(E); free(x); free(y);
    }
    {
        const int64_t dims[3] = {5, 66, 3};
        double a[5 * 66 * 3], r[5 * 66 * 3], c[4], trace[5], margins[12];  /* order * w tie margins */
        int32_t iters[4];
        uint64_t s0[4 * 1], s1[4 * 2], s2[4 * 1];
        uint64_t* so[3] = {s0, s1, s2};
        for (int i = 0; i < 5 * 66 * 3; ++i) a[i] = noise(&st);
        scdo_tensor_decompose(a, 3, dims, 4, 9, 64, so, c, trace, iters, margins, r);
        const uint64_t* sg[3] = {s0, s1, s2};
        scdo_expand(3, dims, 4, sg, c, r);
        if (!(trace[4] <= trace[0])) return 5;
        if (scdo_tensor_lsq_decompose(a, 3, dims, 4, 9, 64, so, c, trace, iters, margins) < 0) return 6;
        double cv[4 * 3];
        scdo_scalars_decompose(a, 3, dims, 4, 9, 64, so, cv, trace, iters, margins);
        if (!(trace[4] <= trace[0])) return 7;
    }
    return 0;
}
