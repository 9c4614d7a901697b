/*
 * randes_place.h -- where the stacks of a serving set-up lie in device memory.
 *
 * Not part of the method and never needed for correct results: the calls of randes.h take any
 * pointers.  Measured on MI355X, device memory falls into a few large groups of addresses, and a
 * kernel whose read and write streams lie in the same group runs several per cent slower than one
 * whose streams lie in different groups; the streaming kernels of randes.h follow suit (retrieve is
 * fastest with both read streams in one group and its output spread over two others, merge with the
 * superposed stack in a group that holds no delta).  Nothing in the runtime reports the groups, so
 * they are found by timing plain copies between the chunks of one large allocation of the caller's,
 * and the stacks are then packed into that allocation accordingly.
 *
 * All arrays are host arrays; `arena` is a device pointer.  Return values and error text as in
 * randes.h.  The two planning calls are pure functions of their arguments and need no device.
 */
#ifndef RANDES_PLACE_H
#define RANDES_PLACE_H

#include <stdint.h>

#include "randes.h"   /* error codes */

#ifdef __cplusplus
extern "C" {
#endif

/* rate(r, w, ctx): measured rate (any unit, larger = faster) of a plain copy that reads chunk r
 * and writes chunk w of the allocation. */
typedef double (*randes_copy_rate_fn)(int32_t read_chunk, int32_t write_chunk, void *ctx);

/* Label every chunk 0 .. n_chunks-1 with a group number 0, 1, ... (labels_out[n_chunks]).
 * Chunks that copy slowly from a reference chunk are in its group, the others are not; the rest is
 * split again from a new reference, until the rates no longer fall into two clusters at least
 * min_separation (relative; <= 0 selects 0.02) apart or max_groups (<= 0 selects 4) groups exist.
 * Groups come in long runs, so a majority vote over five neighbouring chunks removes single
 * misreads.  `rate` is called about n_chunks times per group found.
 * Errors: RANDES_EINVAL (n_chunks < 1, NULL pointers). */
int randes_place_classify(int32_t n_chunks, randes_copy_rate_fn rate, void *ctx,
                          double min_separation, int32_t max_groups, int32_t *labels_out);

/* The same with the rates measured here: best of four timed plain copies (after one that warms up)
 * of chunk r to chunk w of the device allocation [arena, arena + n_chunks * chunk_bytes), on
 * hip_stream, which is synchronised.  chunk_bytes must be a multiple of 16384 and arena 16-byte
 * aligned; the pages of the allocation should have been touched before, and the allocation's
 * contents are overwritten.  About one second for 274 chunks of 1 GiB.
 * Errors: RANDES_EINVAL, RANDES_EHIP. */
int randes_place_classify_device(void *arena, uint64_t chunk_bytes, int32_t n_chunks, void *hip_stream,
                                 int32_t *labels_out);

/* Byte offsets, inside the classified allocation, of the stacks of one serving set-up of
 * n_models models: the superposed stack and the base in one group; the output stack across a
 * boundary between two other groups, half on either side; the models' delta stacks, then
 * n_more_outputs further output stacks, in what is left of every group but the first.  Every stack
 * is contiguous, 256-byte aligned, stack_bytes long, and stays one chunk away from the other group
 * boundaries, whose position is only known to one chunk.
 * offsets_out[3 + n_models + n_more_outputs] = merged, base, out, deltas..., further outputs...;
 * groups_out[3] = the group read by retrieve, and the two groups the output stack lies in.
 * Errors: RANDES_EINVAL; RANDES_ENOTSUP when the groups found do not allow this layout (fewer than
 * three groups, or not enough room): the caller then allocates as it likes. */
int randes_place_serving_layout(const int32_t *labels, int32_t n_chunks, uint64_t chunk_bytes,
                                uint64_t stack_bytes, int32_t n_models, int32_t n_more_outputs,
                                uint64_t *offsets_out, int32_t *groups_out);

#ifdef __cplusplus
}
#endif
#endif /* RANDES_PLACE_H */
