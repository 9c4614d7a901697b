/*
 * randes.h -- C ABI of the RanDeS (Randomized Delta Superposition) hot path
 * on AMD MI355X (gfx950).
 *
 * The two calls a user makes are the paper's problem statement (Sec. "Problem
 * setup"):  Theta_* = compress({Theta_i}),  hat Theta_i = retrieve(Theta_*, i).
 * compress superposes the T deltas Delta_i = Theta_i - Theta_0 after a
 * per-model random orthogonal transform O_i defined by a seed (Sec. 4);
 * O_i is realised layer-wise as a shuffle of same-type layers (Sec. 4.3)
 * followed by a random column-wise sign flip (Sec. 4.4).  No mask or
 * permutation is ever stored: both are regenerated from (seed, layer, column)
 * with the counter-based Philox4x32-10 generator.
 *
 * General rules for every entry point
 *  - Return value: RANDES_OK (0) or a negative error code.  Nothing aborts or
 *    throws.  Arguments are validated before anything is enqueued, so a call
 *    that fails validation writes nothing.
 *  - Pointer arrays (deltas, merged, base, out) are HOST arrays whose entries
 *    are DEVICE pointers.  Every buffer is allocated, owned and freed by the
 *    caller.  The library allocates only small descriptor tables of its own
 *    (cached per distinct argument set, released by randes_shutdown()).
 *  - Layout: a layer is a dense row-major rows x cols matrix, cols contiguous.
 *    "Column" (the index the sign flip acts on, Sec. 4.4) is the contiguous
 *    index.  Rows of one layer are contiguous (no padding between rows).
 *  - Work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream).  Calls do not synchronise; results are valid once
 *    the caller has synchronised the stream.  Buffers must stay alive until
 *    then.  The first call with a given argument set builds its tables on the
 *    host and uploads them synchronously (hipMalloc + hipMemcpy); a repeated
 *    call only launches kernels and may therefore be recorded into a HIP
 *    graph.  A first call made while its stream is being captured is refused
 *    with RANDES_ENOTSUP before anything is enqueued (call once eagerly
 *    first).  256 argument sets stay cached per process; beyond that the least
 *    recently used one is dropped from the cache.  Its tables are released
 *    later: once 64 MiB of dropped tables have collected, a first call (which
 *    allocates and copies synchronously anyway) drains the device and frees
 *    those that no caller still holds; randes_shutdown() frees the rest.  A
 *    cached call never frees, synchronises or allocates.  Tables of a call made
 *    while its stream was being captured are kept until randes_shutdown(),
 *    because the graph's kernels point into them (at most 4096 such sets).
 *  - Threads: every entry point may be called from several host threads at
 *    once; the cache is locked only while a table set is looked up or added,
 *    never across planning, uploads or launches.
 *  - When the tables of an argument set are built (its first call), every
 *    buffer is checked against the HIP runtime's records: it must be memory
 *    HIP knows, not memory of another device than the current one, and its
 *    allocation must hold all rows x cols elements of its layer; otherwise
 *    RANDES_EINVAL, before anything is enqueued.  Cached calls skip the check
 *    (freeing a buffer and calling again with its stale pointer is the
 *    caller's error).  randes_sign_mask and randes_delta_stats_noalloc, which
 *    build no cached tables, do not check.
 *  - Layer pointers must be aligned to their element size (else RANDES_EINVAL).
 *    16-byte aligned layers whose cols is a multiple of 4 (f32) / 8 (bf16)
 *    take the vectorised kernels; anything else takes a slower element-wise
 *    kernel with identical results.
 */
#ifndef RANDES_H
#define RANDES_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RANDES_OK 0
#define RANDES_EINVAL (-1)   /* bad argument (null pointer, size < 1, unknown dtype, mismatched group, non-finite lambda) */
#define RANDES_ENOTSUP (-2)  /* valid request this build does not cover (e.g. n_tasks above RANDES_MAX_TASKS) */
#define RANDES_EHIP (-3)     /* HIP runtime failure; randes_strerror() carries the runtime's text */

#define RANDES_MAX_TASKS 128

typedef enum { RANDES_F32 = 0, RANDES_BF16 = 1 } randes_dtype;

/* Per-layer flags.  FLIP: the layer takes the random sign flip D (Sec. 4.4).
 * SHUFFLE: the layer takes part in its group's random permutation (Sec. 4.3).
 * SHIFT: the group is rotated instead of shuffled, the layer-shifting variant of
 * App. "Dynamics between Layer Shuffling and Random Sign Flips": model `seed`
 * has every member moved (seed mod G) + 1 slots deeper, cyclically, so models
 * with consecutive seeds lie one slot apart.
 * flags = 0 is the Identity context of Sec. "Impact of Context Matrix Design",
 * i.e. plain task arithmetic; choosing which layers carry flags realises the
 * ALL / MLP / ATTN target selection and the target-layer skip rate. */
enum { RANDES_FLIP = 1, RANDES_SHUFFLE = 2, RANDES_SHIFT = 4 };

/* One parameter matrix Delta^{k,j} in R^{m x n} (Sec. 4.2 "Layer-wise Notation").
 * group: id of the set {Delta^{k,j}}_k of same-type layers across blocks;
 * negative = belongs to no group (input / output layers).  The k-th member of
 * a group is the k-th layer, in ascending index, that carries the group id and
 * RANDES_SHUFFLE or RANDES_SHIFT; all members must have equal rows and cols.
 * The group id itself is fed to the generator, so renumbering groups changes
 * the permutations. */
typedef struct {
    int64_t rows;   /* m >= 1 */
    int64_t cols;   /* n >= 1, n < 2^31 */
    int32_t group;
    int32_t flags;
} randes_layer;

/* Permutation sigma ~ S_G of one (model, group) pair (Sec. 4.3).  HOST only,
 * needs no GPU.  perm_out[k] = sigma(k) = within-group index of the layer that
 * lands in slot k (Delta^{k,j} <- Delta^{sigma(k),j}).  perm_out: host array of
 * group_size int32.  sigma is the stable ascending argsort of 64-bit keys drawn
 * from Philox4x32-10 at counter (k, group, 1, 0) under key (seed low, seed high).
 * Errors: RANDES_EINVAL if perm_out is NULL or group_size < 1. */
int randes_layer_perm(uint64_t seed, int32_t group, int32_t group_size, int32_t *perm_out);

/* Whole-model form of the above.  HOST only.  src_out[l] = index of the layer
 * of this model whose delta lands in slot l (identity for layers outside any
 * shuffled group).  src_out: host array of n_layers int32.
 * Errors: RANDES_EINVAL on null pointers, n_layers < 1, bad layer sizes, or a
 * group whose members differ in shape (the size mismatch Sec. 4.3 rules out). */
int randes_source_table(const randes_layer *layers, int32_t n_layers, uint64_t seed, int32_t *src_out);

/* Diagonal of the context matrix D of one (model, slot layer) pair (Sec. 4.4:
 * entries +1 / -1 with equal probability), as the device kernels regenerate it.
 * mask_out: DEVICE array of cols bytes; mask_out[c] = 1 where D_cc = -1, else 0.
 * Bit (c mod 32) of word ((c / 32) mod 4) of Philox4x32-10 at counter
 * (c / 128, layer, 0, 0) under key (seed low, seed high). */
int randes_sign_mask(uint64_t seed, int32_t layer, int64_t cols, uint8_t *mask_out, void *hip_stream);

/* compress (Sec. 4, first display; layer-wise: Sec. 4.3 then Sec. 4.4):
 *   merged[l][r][c] = sum_{i=0}^{n_tasks-1} (-1)^{s(seeds[i], l, c)} * deltas[i][src_i(l)][r][c]
 * accumulated in binary32 starting from +0 in task order i = 0, 1, ...; stored
 * as merged_dtype (bf16: round to nearest even).  lambda is NOT folded in; it is
 * applied at retrieval.
 *   layers    host array of n_layers descriptors
 *   deltas    host array of n_tasks * n_layers device pointers;
 *             deltas[i * n_layers + l] = model i's layer l in its ORIGINAL position
 *   seeds     host array of n_tasks per-model seeds (App. "Default Experimental
 *             Setup": global seed + model index)
 *   merged    host array of n_layers device pointers (outputs; must not alias any delta)
 * Errors: RANDES_EINVAL (see above), RANDES_ENOTSUP (n_tasks > RANDES_MAX_TASKS),
 * RANDES_EHIP. */
int randes_merge(const randes_layer *layers, int32_t n_layers,
                 const void *const *deltas, int32_t n_tasks, const uint64_t *seeds,
                 randes_dtype delta_dtype,
                 void *const *merged, randes_dtype merged_dtype, void *hip_stream);

/* compress straight from the fine-tuned weights: the delta Delta_i = Theta_i - Theta_0 (Sec. 3) is
 * formed on the fly in binary32 (one rounding, never rounded to the storage dtype), so no delta
 * buffers are needed:
 *   merged[l][r][c] = sum_i (-1)^{s(seeds[i], l, c)} * (weights[i][src_i(l)][r][c] - base[src_i(l)][r][c])
 * otherwise exactly as randes_merge.  weights: host array of n_tasks * n_layers device pointers
 * (model i's layer l at [i * n_layers + l]); base: host array of n_layers device pointers; both of
 * weight_dtype.  For f32 weights the result equals randes_merge on f32 deltas computed as Theta_i - Theta_0. */
int randes_merge_weights(const randes_layer *layers, int32_t n_layers,
                         const void *const *weights, const void *const *base, int32_t n_tasks, const uint64_t *seeds,
                         randes_dtype weight_dtype, void *const *merged, randes_dtype merged_dtype, void *hip_stream);

/* retrieve (Sec. 4, second display; Sec. 4.4 with D^-1 = D; Sec. 4.3 inverse permutation):
 * slot l of the superposition goes back to layer t = src(l) of the requested model,
 *   out[t][r][c] = fma(lambda, (-1)^{s(seed, l, c)} * merged[l][r][c], base[t][r][c])
 * one rounding in binary32, stored as out_dtype (bf16: round to nearest even).
 *   merged, base, out   host arrays of n_layers device pointers
 *   out[l] may be the same buffer as base[l]; out must not alias merged.
 * Errors: RANDES_EINVAL (also for NaN / Inf lambda), RANDES_EHIP. */
int randes_retrieve(const randes_layer *layers, int32_t n_layers,
                    const void *const *merged, randes_dtype merged_dtype,
                    const void *const *base, randes_dtype base_dtype,
                    uint64_t seed, float lambda,
                    void *const *out, randes_dtype out_dtype, void *hip_stream);

/* retrieve for several models in one pass over the superposition (the retrieval of Sec. 4 applied
 * n_requests times; "retrieve(Theta*, i)" of the problem setup for a batch of i): for request q,
 *   outs[q][t_q][r][c] = fma(lambdas[q], (-1)^{s(seeds[q], l, c)} * merged[l][r][c], base[t_q][r][c]),  t_q = src_q(l)
 * every output stack bit-identical to what randes_retrieve gives for (seeds[q], lambdas[q]).
 * When merged, base and outs share one dtype and every layer is 16-byte aligned with cols a
 * multiple of 4 (f32) / 8 (bf16), requests are served 8, 4 or 2 at a time by a kernel that reads
 * each merged tile once for all of them (2 + 4 q bytes per element and q requests in bf16 instead
 * of 6 q); otherwise, and for a request left over, the call runs randes_retrieve per request.
 *   seeds, lambdas   host arrays of n_requests
 *   outs             host array of n_requests * n_layers device pointers; outs[q * n_layers + l] =
 *                    request q's layer l.  Output stacks must not overlap each other, merged or base
 *                    (unlike randes_retrieve, base is read by every request of a pass).
 * Errors: RANDES_EINVAL (also n_requests < 1, NaN / Inf lambda, overlapping outputs), RANDES_EHIP. */
int randes_retrieve_many(const randes_layer *layers, int32_t n_layers,
                         const void *const *merged, randes_dtype merged_dtype,
                         const void *const *base, randes_dtype base_dtype,
                         int32_t n_requests, const uint64_t *seeds, const float *lambdas,
                         void *const *outs, randes_dtype out_dtype, void *hip_stream);

/* Hot swap (Sec. "Model Hot Swapping"): add (remove = 0) or remove (remove != 0)
 * one model in place, without touching the others:
 *   merged[l][r][c] <- merged[l][r][c] +/- (-1)^{s(seed, l, c)} * delta[src(l)][r][c]
 * one binary32 addition per element, stored back as merged_dtype.  With f32
 * storage, adding a model is bit-identical to having merged it last.
 *   delta   host array of n_layers device pointers (original positions) */
int randes_update(const randes_layer *layers, int32_t n_layers,
                  void *const *merged, randes_dtype merged_dtype,
                  const void *const *delta, randes_dtype delta_dtype,
                  uint64_t seed, int32_t remove, void *hip_stream);

/* Diagnostics of Sec. 3 ("Interference in Model Merging") on the device: inner product and squared
 * norms of two transformed deltas over a whole stack, in binary64,
 *   a'[l] = D_a^l-flipped delta_a[src_a(l)],   b'[l] = D_b^l-flipped delta_b[src_b(l)]
 *   out3 = { <a', b'>, <a', a'>, <b', b'> }          (out3: DEVICE array of 3 doubles)
 * from which follow the pairwise cosine similarity of (interfering) deltas and the interference norm
 * identity || sum_j Delta_j ||^2 = sum_j ||Delta_j||^2 + 2 sum_{l<j} <Delta_l, Delta_j>.  Pass layers with
 * flags = 0 for the untransformed deltas.  The common factor D_i^-1 of a retrieval is orthogonal and
 * drops out of every inner product, so it is not needed here.  Work proceeds through per-workgroup
 * partial sums summed in a fixed order, so the result is reproducible.  The partial sums live beside
 * the cached tables, one set per (argument set, stream): calls on one stream run in order, and equal
 * calls on different streams do not share them.  (So the eager call that must precede recording this
 * call into a graph has to be made on the stream that is then captured.) */
int randes_delta_stats(const randes_layer *layers, int32_t n_layers,
                       const void *const *delta_a, uint64_t seed_a,
                       const void *const *delta_b, uint64_t seed_b,
                       randes_dtype dtype, double *out3, void *hip_stream);

/* randes_delta_stats for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * result, bit for bit, as randes_delta_stats; the call consists of kernel launches only (no
 * hipMalloc, hipFree or hipMemcpy, nothing cached).  The descriptor tables of the call and its
 * per-workgroup partial sums go to a fixed 8 MiB array inside the library's code object (one copy per
 * GPU, held until the process ends) instead of allocated memory; the tables travel inside kernel
 * arguments.  Limits: the tables must fit 1 MiB (a few thousand layers) and the partial sums 7 MiB
 * (305834 workgroups: about 10^10 bf16 or 5 * 10^9 f32 elements per stack); beyond either the call
 * returns RANDES_ENOTSUP and enqueues nothing.  Nothing in the array needs clearing between calls.
 * Every call on a GPU uses that GPU's one array: calls on the same stream run in order and are safe;
 * calls that overlap in time on different streams of one GPU race on it and must be ordered by the
 * caller. */
int randes_delta_stats_noalloc(const randes_layer *layers, int32_t n_layers,
                               const void *const *delta_a, uint64_t seed_a,
                               const void *const *delta_b, uint64_t seed_b,
                               randes_dtype dtype, double *out3, void *hip_stream);

/* LoRA front-end (Sec. "Parameter Efficient Finetuning (PEFT) Model Compression":
 * Theta_i = Theta_0 + lambda L_i): materialise the dense adapter update
 *   delta_out[r][c] = scale * sum_{t < rank} B[r][t] * A[t][c]
 * on the matrix cores (bf16 or f32 MFMA, binary32 accumulate), so it can enter
 * randes_merge as a delta.  B: device, rows x rank row-major.  A: device,
 * rank x cols row-major.  delta_out: device, rows x cols row-major.
 * rank >= 1 (any value; padded internally to the MFMA depth).
 * The summation order inside the matrix cores is the hardware's; results agree
 * with exact arithmetic to within rank * 2^-24 * sum_t |B||A| (plus the final
 * rounding to out_dtype). */
int randes_lora_materialize(const void *B, const void *A, int64_t rows, int64_t cols, int32_t rank,
                            float scale, randes_dtype ab_dtype,
                            void *delta_out, randes_dtype out_dtype, void *hip_stream);

/* Batched form: n matrices in one launch.  Bs, As, outs: host arrays of n device
 * pointers; rows, cols: host arrays of n sizes; one rank, scale and dtype pair. */
int randes_lora_materialize_batched(int32_t n, const void *const *Bs, const void *const *As,
                                    const int64_t *rows, const int64_t *cols, int32_t rank,
                                    float scale, randes_dtype ab_dtype,
                                    void *const *outs, randes_dtype out_dtype, void *hip_stream);

/* Fused LoRA compress (Sec. "Parameter Efficient Finetuning (PEFT) Model Compression" + Sec. 4.3 / 4.4):
 * superpose T adapters without materialising any of them,
 *   merged[l] = scale * sum_i B_i[src_i(l)] A_i[src_i(l)] D_i^l
 *             = scale * [B_1 .. B_T] [A_1 D_1; ..; A_T D_T]        (one rank T*r contraction per layer)
 * on the matrix cores with binary32 accumulation, rounded once to merged_dtype.
 *   layers   the adapter-carrying matrices only (rows x cols of the dense update), with flags and groups
 *   Bs, As   host arrays of n_tasks * n_layers device pointers, [i * n_layers + l] = model i's factors of
 *            layer l (original position); B is rows x rank, A is rank x cols, row-major
 * Differs from materialise-then-merge only by rounding: no intermediate rounding of each L_i to the
 * storage dtype, and the matrix cores' own summation order. */
int randes_lora_merge(const randes_layer *layers, int32_t n_layers,
                      const void *const *Bs, const void *const *As, int32_t rank,
                      int32_t n_tasks, const uint64_t *seeds, float scale, randes_dtype ab_dtype,
                      void *const *merged, randes_dtype merged_dtype, void *hip_stream);

/* Text for an error code; for RANDES_EHIP the text of the last HIP failure seen
 * by the calling thread.  Never NULL; valid until the thread's next failing call. */
const char *randes_strerror(int code);

/* Free every cached descriptor table on every device.  The caller must have
 * synchronised all streams that ran library work.  Safe to call repeatedly. */
int randes_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* RANDES_H */
