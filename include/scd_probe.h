/*
 * scd_probe.h -- measurement instruments of libscd.so.  Not part of the method's interface (scd.h): these
 * calls exist so that the benchmark and the profiles can time single kernels and the chip's own ceilings.
 * Same conventions as scd.h (device pointers unless documented "host", status codes, void* streams).
 */
#ifndef SCD_PROBE_H
#define SCD_PROBE_H

#include "scd.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Sparse engine only (zeros otherwise): how many row signs and column signs changed after the first
 * alternation of their term, summed over the terms run so far.  Section 3.1's cached products re-read one
 * row of R per changed row sign and one column per changed column sign: these counts give the bytes the
 * paper's own method moves (host pointers, may be NULL). */
int scd_sparse_flips(const scd_ctx* ctx, int64_t* row_flips, int64_t* col_flips);

/* Algorithmic bytes the row-pass kernels of this context have read+written so far and the number
 * of passes (launches) they took: the counters behind the bandwidth figures.  host pointers. */
int scd_traffic(const scd_ctx* ctx, double* bytes, int64_t* passes, int64_t* sweeps);

/* Which engine scd_run uses for this context: 0 = a stream of launches that re-read the remainder from
 * memory every alternation (any shape, dtype, order); 1 = one persistent launch that keeps the whole
 * remainder in the register files of a grid of workgroups (f32 matrices that fit, see SCD_OPT_RESIDENT);
 * 2 = one persistent launch that caches R t and R^T s and updates them from the flipped signs only
 * (Section 3.1; f32/f64 matrices with 8 <= m, n <= 65536 whose rows and columns are multiples of 16 bytes and
 * whose remainder takes at least SCD_OPT_SPARSE_MIN_MIB, or any size once the context has a share of the
 * device; keeps a transposed copy of the remainder; finished terms wait in a list of SCD_OPT_SPARSE_DELAY_WIDTH
 * before they are subtracted, Section 3.2.  With delayed updates ||R_k||_F is measured from the remainder at
 * every flush of the list and at the end of every scd_run; between flushes it follows Section 3.2's identity
 * ||R - c s t^T||^2 = ||R||^2 - 2 c <s, R t> + c^2 mn from the cut value); 3 = one persistent launch that
 * streams the remainder from memory once per alternation (matrices whose rows are a multiple of 16 bytes and at
 * most 64 KB long; the first rows of every workgroup's block stay in LDS).  For engines 1, 2 and 3 also the
 * duration of the most recent launch by HIP events on the context's stream and its dense-equivalent bytes:
 * (alternations + updates) * bytes of the remainder, what a streaming pass per alternation would move.  host
 * pointers, each may be NULL. */
int scd_engine(const scd_ctx* ctx, int* engine, double* last_launch_seconds, double* last_launch_bytes);

/* The launch geometry the persistent streaming engine would use for an array of this dtype and shape on at most
 * `limit` workgroups (host arrays; no GPU work): out[0] = 1 if the engine takes the shape (else 0 and the rest is
 * unspecified), out[1] workgroups, out[2] rows per workgroup, out[3] columns per slice of the first exchange,
 * out[4] rows of a block kept in LDS, out[5] bytes of dynamic LDS, out[6] / out[7] bytes of the two exchange
 * buffers.  For tests of the host arithmetic against the bounds the kernel assumes. */
int scd_stream_geometry(scd_dtype dt, int order, const int64_t* dims, int limit, int64_t out[8]);

/* Measurement: run n (<= 4096) further sweeps of the greedy loop with a HIP event before and after
 * each kernel of the pass over the remainder; returns the average duration of the row-pass launch
 * and of the reduce launch that follows it (host pointers, seconds).  The terms found meanwhile are
 * ordinary terms of the decomposition; SCD_EFULL if the context is at capacity. */
int scd_profile_sweeps(scd_ctx* ctx, int n, double* rowpass_seconds, double* reduce_seconds);

/* Plain streaming kernels, for measurement only.  dst == NULL: read `bytes` (a multiple of 16) from
 * src and discard them; else copy src to dst.  `grid` workgroups of 256 threads, one untimed launch
 * and then `reps` timed ones; *seconds (host) = average time of one launch by HIP events on `stream`.
 * The read rate of a buffer that is re-read gives the ceiling of the cache-resident row pass; the
 * copy of known size calibrates the memory counters of the profiler. */
int scd_probe_stream(const void* src, void* dst, int64_t bytes, int grid, int reps, void* stream,
                     double* seconds);

/* Latency of exchanging data between the workgroups of one persistent launch, for measurement only.
 * which = 0: every workgroup publishes 256 tagged values per round and reads those of its `group`
 * neighbours (the exchange the register-resident engine uses); which = 1: a counter barrier over the
 * whole grid.  grid workgroups (a multiple of group, at most 1024; keep it at most the number of
 * compute units) must all be resident at once; every wait is bounded and SCD_EINVAL is returned when
 * one runs out.  *seconds_per_round: host. */
int scd_probe_exchange(int which, int grid, int group, int rounds, void* stream, double* seconds_per_round);

#ifdef __cplusplus
}
#endif
#endif /* SCD_PROBE_H */
