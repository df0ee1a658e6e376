/*
 * sar_bench_probes.h -- bandwidth probes for bench.py (libsar_bench.so).
 *
 * Not part of the method and not part of the product library: plain kernels that
 * measure the ceilings the aggregation kernels are held against on the machine at
 * hand (the paper reports its kernels only relative to another library, Sec. 4.1;
 * these give an absolute yardstick).  Every pointer is a device pointer owned by the
 * caller; `stream` is a hipStream_t; calls only enqueue work and the caller times
 * them with events on that stream.  Return 0, or -1 (invalid argument), -2
 * (unsupported row size), -3 (launch failed).  sink: device float[1].
 */
#ifndef SAR_BENCH_PROBES_H
#define SAR_BENCH_PROBES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Reads `bytes` at buf `reps` times with 16-byte lane accesses, grid-stride. */
int sar_bench_stream_read(const void* buf, size_t bytes, int reps, float* sink, void* stream);

/* dst[0..bytes) = src[0..bytes). */
int sar_bench_copy(const void* src, void* dst, size_t bytes, void* stream);

/* For every k < n_idx (in groups of 8 per wavefront) reads the whole row rows[idx[k]] of
 * row_bytes (1024 or 512) bytes; idx values must be in [0, n_rows).  The access shape of the
 * aggregation kernels without their arithmetic. */
int sar_bench_row_gather(const void* rows, int64_t n_rows, int row_bytes, const int32_t* idx,
                         int64_t n_idx, float* sink, void* stream);

/* The same gathers with writes mixed in: after every 8 gathered rows, writes_per_8 (0..8) of them
 * are written to consecutive rows of out, which must hold (n_idx / 8) * writes_per_8 rows.  The
 * read/write mix of the backward kernels without their arithmetic. */
int sar_bench_gather_write(const void* rows, int64_t n_rows, int row_bytes, const int32_t* idx,
                           int64_t n_idx, int writes_per_8, void* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SAR_BENCH_PROBES_H */
