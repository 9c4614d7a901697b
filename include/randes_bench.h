/*
 * randes_bench.h -- measurement aids of librandes.so.  Nothing here belongs to the method: these
 * calls exist so that a benchmark can vary the launch shape of the streaming kernels and can time a
 * plain streaming kernel of the same shape on the same buffers.  Results of the calls declared in
 * randes.h never depend on the knobs.  The knobs are per host thread: they shape the calls made by
 * the thread that set them and nobody else's.
 */
#ifndef RANDES_BENCH_H
#define RANDES_BENCH_H

#include <stdint.h>

#include "randes.h"   /* error codes */

#ifdef __cplusplus
extern "C" {
#endif

/* Launch-shape knob: rows of a tile that one wavefront owns (0 = built-in default: the kernels'
 * burst size for merge and the diagnostics, a share of it chosen by the size of the stack for
 * retrieve and hot swap; values above the burst size are clamped to it).  Results never depend on
 * them.  Returns RANDES_EINVAL for negative values. */
int randes_set_tile_rows(int32_t merge_rows, int32_t retrieve_rows);

/* Second launch-shape knob: how many of a workgroup's 4 wavefronts may sit side by
 * side along the columns (4, 2 or 1; 0 = default 4); the rest stack along the rows.
 * Results never depend on it. */
int randes_set_tile_cols(int32_t max_waves_along_columns);

/* Third launch-shape knob: a layer whose row length leaves lanes of the column tiles idle (768
 * bf16 columns: a quarter of them) is handed to the kernels with 2..8 consecutive rows shown as
 * one longer row (rows are contiguous in memory; the sign pattern of Sec. 4.4 then simply repeats
 * along the longer row).  enable = 0 switches this off (default on).  Results never depend on it. */
int randes_set_fold(int32_t enable);

/* Measurement aid, not part of the method: a plain streaming kernel with the same
 * launch shape as merge / retrieve and nothing else in it.  Reads n_inputs (1..8)
 * device streams of `bytes` bytes each (16-byte aligned, bytes a multiple of 16384)
 * and, if write != 0, stores their element-wise 32-bit integer sum to output
 * (bytes bytes); if write == 0 nothing is stored and output only needs 16 valid
 * bytes.  Its bandwidth is a point of comparison for that mix of reads and writes
 * (one plain kernel of one launch shape, not an upper bound), reported beside the
 * method's kernels by the benchmark. */
int randes_probe_stream(const void *const *inputs, int32_t n_inputs, void *output, int64_t bytes, int32_t write,
                        void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RANDES_BENCH_H */
