/*
 * RanDeS CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, deliberately unoptimised implementation of the RanDeS
 * (Randomized Delta Superposition) compress / retrieve path, written from the
 * paper (Sec. 4 "Randomized Delta Superposition", Sec. 4.3 "Layer Shuffling",
 * Sec. 4.4 "Layer Column-wise Random Sign Flips", App. "Default Experimental
 * Setup").  It exists so that the GPU library can be checked against it.  It
 * shares no code, header, table or helper with the GPU library and must never
 * be called from a product path: only tests, the smoke check and the
 * benchmark's CPU-baseline leg may load it.
 *
 * Every function below is pinned by a CPU-only test against something other
 * than itself (published known-answer vectors of the generator, closed forms,
 * invariants, dense brute force).  Nothing here is "parity unpinned".
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (no intrinsics).
 *
 * Conventions (paper notation): T fine-tuned models ("tasks", here n_tasks),
 * Theta_0 base weights, Delta_i = Theta_i - Theta_0 the delta of model i,
 * lambda the merging coefficient, a "layer" is one parameter matrix
 * Delta_i^{k,j} in R^{m x n} stored row-major (n contiguous).  A shuffle group
 * is the set {Delta_i^{k,j}}_k of same-type layers across blocks.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_F32 0
#define ORACLE_BF16 1

#define ORACLE_FLIP 1    /* layer takes the random column sign flip   */
#define ORACLE_SHUFFLE 2 /* layer takes part in its group's shuffle   */
#define ORACLE_SHIFT 4   /* group is rotated deeper instead of shuffled */

typedef struct {
    int64_t rows;  /* m */
    int64_t cols;  /* n: the contiguous index, the one the sign flip acts on */
    int32_t group; /* shuffle group id; < 0 = not in any group */
    int32_t flags;
} oracle_layer;

/* ------------------------------------------------------------------------
 * Philox4x32-10, the counter-based generator of Salmon, Moraes, Dror & Shaw
 * (SC'11).  The paper names no generator (App. "Default Experimental Setup"
 * only fixes seeds); this one is chosen because any (seed, layer, column) can
 * be evaluated independently.  One round: two 32x32->64 products of counter
 * words 0 and 2 with the multipliers below; the high halves are xored with
 * counter words 1 and 3 and the round key; the key is then advanced by the
 * Weyl constants.
 * ---------------------------------------------------------------------- */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------
 * Sign of the context matrix D_i^{l} (Sec. 4.4: diagonal, entries +1 / -1
 * with equal probability).  s = 1 means D_cc = -1.  The stream is indexed by
 * (model seed, slot layer l, column c): one generator call yields the 128
 * sign bits of columns [128*b, 128*b+128), bit (c mod 32) of word
 * ((c / 32) mod 4).
 * ---------------------------------------------------------------------- */
uint32_t oracle_sign_bit(uint64_t seed, uint32_t layer, uint64_t col)
{
    uint32_t ctr[4] = { (uint32_t)(col / 128u), layer, 0u, 0u };
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    uint32_t word = out[(col / 32u) % 4u];
    return (word >> (col % 32u)) & 1u;
}

/* mask_out[c] = sign bit of column c, for c in [0, cols). */
void oracle_sign_mask(uint64_t seed, uint32_t layer, int64_t cols, uint8_t *mask_out)
{
    for (int64_t c = 0; c < cols; ++c)
        mask_out[c] = (uint8_t)oracle_sign_bit(seed, layer, (uint64_t)c);
}

/* ------------------------------------------------------------------------
 * Layer permutation sigma ~ S_G (Sec. 4.3).  Each position k draws a 64-bit
 * sort key from the generator at counter (k, group, 1, 0); sigma is the
 * stable ascending argsort of those keys, so perm_out[k] = sigma(k) is the
 * within-group index of the layer that lands in slot k.  Distinct keys give a
 * uniformly random permutation; ties (probability ~ G^2 / 2^65) fall back to
 * position order.  keys_out may be NULL.
 * ---------------------------------------------------------------------- */
void oracle_layer_perm(uint64_t seed, int32_t group, int32_t group_size,
                       int32_t *perm_out, uint64_t *keys_out)
{
    uint32_t key[2] = { (uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32) };
    uint64_t *keys = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)(group_size > 0 ? group_size : 1));
    for (int32_t k = 0; k < group_size; ++k) {
        uint32_t ctr[4] = { (uint32_t)k, (uint32_t)group, 1u, 0u };
        uint32_t out[4];
        oracle_philox4x32_10(ctr, key, out);
        keys[k] = ((uint64_t)out[0] << 32) | (uint64_t)out[1];
        if (keys_out) keys_out[k] = keys[k];
        perm_out[k] = k;
    }
    /* insertion sort: stable, and G is the number of blocks (tens) */
    for (int32_t a = 1; a < group_size; ++a) {
        int32_t p = perm_out[a];
        int32_t b = a - 1;
        while (b >= 0 && keys[perm_out[b]] > keys[p]) {
            perm_out[b + 1] = perm_out[b];
            --b;
        }
        perm_out[b + 1] = p;
    }
    free(keys);
}

/* ------------------------------------------------------------------------
 * Number formats.  bf16 is the upper half of an IEEE binary32; widening is
 * exact; narrowing rounds to nearest, ties to even; NaN stays a quiet NaN.
 * ---------------------------------------------------------------------- */
static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

float oracle_bf16_to_f32(uint16_t h) { return bits_to_f32((uint32_t)h << 16); }

uint16_t oracle_f32_to_bf16(float f)
{
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) /* NaN */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t lower = u & 0xffffu;      /* the part that is dropped */
    uint32_t upper = u >> 16;
    if (lower > 0x8000u || (lower == 0x8000u && (upper & 1u)))
        upper += 1u;                   /* carries into the exponent correctly */
    return (uint16_t)upper;
}

static float load_elem(const void *p, int64_t idx, int dtype)
{
    if (dtype == ORACLE_F32) return ((const float *)p)[idx];
    return oracle_bf16_to_f32(((const uint16_t *)p)[idx]);
}

static void store_elem(void *p, int64_t idx, int dtype, float v)
{
    if (dtype == ORACLE_F32) ((float *)p)[idx] = v;
    else ((uint16_t *)p)[idx] = oracle_f32_to_bf16(v);
}

/* ------------------------------------------------------------------------
 * Source table.  src_out[i * n_layers + l] = index of the layer of model i
 * whose delta lands in slot l after model i's shuffle (Sec. 4.3:
 * Delta_i^{k,j} <- Delta_i^{sigma_i^j(k), j}).  The members of group g are
 * the layers carrying that group id and the SHUFFLE (or SHIFT) flag, in
 * ascending layer order; everything else stays in place.  SHIFT replaces the
 * random permutation by the deterministic layer shifting of App. "Dynamics
 * between Layer Shuffling and Random Sign Flips" (every layer moves deeper,
 * the deepest ones wrapping round to the front).  The appendix reports that
 * shifting changes the cosine similarity among interfering deltas, which a
 * rotation common to all models cannot do (it would only relabel the slots),
 * so the distance depends on the model: model `seed` is rotated by
 * d = (seed mod G) + 1 positions, taken mod G; slot (k + d) mod G receives
 * layer k.  Seed 0 moves by one position and consecutive seeds (App. "Default
 * Experimental Setup": global seed + model index) lie one position apart.
 * Returns 0, or -1 if members of one group differ in shape.
 * ---------------------------------------------------------------------- */
int oracle_source_table(const oracle_layer *layers, int32_t n_layers,
                        const uint64_t *seeds, int32_t n_tasks, int32_t *src_out)
{
    int32_t *members = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers);
    int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers);
    char *done = (char *)calloc((size_t)n_layers, 1);
    int rc = 0;
    for (int32_t i = 0; i < n_tasks; ++i)
        for (int32_t l = 0; l < n_layers; ++l)
            src_out[(int64_t)i * n_layers + l] = l;
    for (int32_t l = 0; l < n_layers && rc == 0; ++l) {
        int movable = (layers[l].flags & (ORACLE_SHUFFLE | ORACLE_SHIFT)) != 0;
        if (done[l] || layers[l].group < 0 || !movable) continue;
        int32_t g = layers[l].group, G = 0;
        int shift = 0;
        for (int32_t q = l; q < n_layers; ++q) {
            if (layers[q].group == g && (layers[q].flags & (ORACLE_SHUFFLE | ORACLE_SHIFT))) {
                if (layers[q].rows != layers[l].rows || layers[q].cols != layers[l].cols) rc = -1;
                if (layers[q].flags & ORACLE_SHIFT) shift = 1;
                members[G++] = q;
                done[q] = 1;
            }
        }
        if (rc) break;
        for (int32_t i = 0; i < n_tasks; ++i) {
            if (shift) {
                int32_t d = (int32_t)((seeds[i] % (uint64_t)G + 1u) % (uint64_t)G);
                for (int32_t k = 0; k < G; ++k) perm[(k + d) % G] = k;
            } else {
                oracle_layer_perm(seeds[i], g, G, perm, NULL);
            }
            for (int32_t k = 0; k < G; ++k)
                src_out[(int64_t)i * n_layers + members[k]] = members[perm[k]];
        }
    }
    free(members); free(perm); free(done);
    return rc;
}

/* ------------------------------------------------------------------------
 * compress (Sec. 4 eq. for Theta_*, realised layer-wise by Sec. 4.3 then
 * Sec. 4.4): for every slot layer l, row r, column c
 *     Delta_*[l][r][c] = sum_{i=0}^{T-1} (-1)^{s(seed_i, l, c)} * Delta_i[src_i(l)][r][c]
 * accumulated in binary32 from +0 in task order i = 0, 1, ..., T-1.
 * deltas[i * n_layers + l] points at model i's layer l in its ORIGINAL
 * position.  Shuffle first, flip second: the mask is keyed by the slot.
 * ---------------------------------------------------------------------- */
int oracle_merge(const oracle_layer *layers, int32_t n_layers,
                 const void *const *deltas, int32_t n_tasks, const uint64_t *seeds,
                 int delta_dtype, void *const *merged, int merged_dtype, int n_threads)
{
    int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers * (size_t)n_tasks);
    if (oracle_source_table(layers, n_layers, seeds, n_tasks, src) != 0) { free(src); return -1; }
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t m = layers[l].rows, n = layers[l].cols;
        uint8_t *sign = (uint8_t *)calloc((size_t)n * (size_t)n_tasks, 1);
        if (layers[l].flags & ORACLE_FLIP)
            for (int32_t i = 0; i < n_tasks; ++i)
                oracle_sign_mask(seeds[i], (uint32_t)l, n, sign + (int64_t)i * n);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < m; ++r) {
            for (int64_t c = 0; c < n; ++c) {
                float acc = 0.0f;
                for (int32_t i = 0; i < n_tasks; ++i) {
                    const void *d = deltas[(int64_t)i * n_layers + src[(int64_t)i * n_layers + l]];
                    float x = load_elem(d, r * n + c, delta_dtype);
                    if (sign[(int64_t)i * n + c]) x = -x;
                    acc = acc + x;
                }
                store_elem(merged[l], r * n + c, merged_dtype, acc);
            }
        }
        free(sign);
    }
    free(src);
    return 0;
}

/* ------------------------------------------------------------------------
 * compress from the fine-tuned weights themselves: the delta of Sec. 3,
 * Delta_i = Theta_i - Theta_0, is formed element by element in binary32 and
 * then treated exactly as in oracle_merge.  weights[i * n_layers + l] and
 * base[l] are in their original positions; both have dtype weight_dtype.
 * ---------------------------------------------------------------------- */
int oracle_merge_weights(const oracle_layer *layers, int32_t n_layers,
                         const void *const *weights, const void *const *base, int32_t n_tasks,
                         const uint64_t *seeds, int weight_dtype, void *const *merged, int merged_dtype,
                         int n_threads)
{
    int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers * (size_t)n_tasks);
    if (oracle_source_table(layers, n_layers, seeds, n_tasks, src) != 0) { free(src); return -1; }
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t m = layers[l].rows, n = layers[l].cols;
        uint8_t *sign = (uint8_t *)calloc((size_t)n * (size_t)n_tasks, 1);
        if (layers[l].flags & ORACLE_FLIP)
            for (int32_t i = 0; i < n_tasks; ++i)
                oracle_sign_mask(seeds[i], (uint32_t)l, n, sign + (int64_t)i * n);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < m; ++r) {
            for (int64_t c = 0; c < n; ++c) {
                float acc = 0.0f;
                for (int32_t i = 0; i < n_tasks; ++i) {
                    const int32_t t = src[(int64_t)i * n_layers + l];
                    float theta = load_elem(weights[(int64_t)i * n_layers + t], r * n + c, weight_dtype);
                    float theta0 = load_elem(base[t], r * n + c, weight_dtype);
                    float x = theta - theta0;
                    if (sign[(int64_t)i * n + c]) x = -x;
                    acc = acc + x;
                }
                store_elem(merged[l], r * n + c, merged_dtype, acc);
            }
        }
        free(sign);
    }
    free(src);
    return 0;
}

/* ------------------------------------------------------------------------
 * retrieve (Sec. 4 eq. for hat Theta_i; Sec. 4.4 with D^{-1} = D; Sec. 4.3:
 * the model's permutation is undone): slot l of the
 * superposition goes back to layer t = src(l) of the requested model:
 *     out[t][r][c] = base[t][r][c] + lambda * ((-1)^{s(seed, l, c)} * Delta_*[l][r][c])
 * with a single rounding (fused multiply-add) in binary32.
 * ---------------------------------------------------------------------- */
int oracle_retrieve(const oracle_layer *layers, int32_t n_layers,
                    const void *const *merged, int merged_dtype,
                    const void *const *base, int base_dtype,
                    uint64_t seed, float lambda,
                    void *const *out, int out_dtype, int n_threads)
{
    int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers);
    if (oracle_source_table(layers, n_layers, &seed, 1, src) != 0) { free(src); return -1; }
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t m = layers[l].rows, n = layers[l].cols;
        const int32_t t = src[l];
        uint8_t *sign = (uint8_t *)calloc((size_t)n, 1);
        if (layers[l].flags & ORACLE_FLIP)
            oracle_sign_mask(seed, (uint32_t)l, n, sign);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < m; ++r) {
            for (int64_t c = 0; c < n; ++c) {
                float y = load_elem(merged[l], r * n + c, merged_dtype);
                if (sign[c]) y = -y;
                float b = load_elem(base[t], r * n + c, base_dtype);
                store_elem(out[t], r * n + c, out_dtype, fmaf(lambda, y, b));
            }
        }
        free(sign);
    }
    free(src);
    return 0;
}

/* ------------------------------------------------------------------------
 * LoRA delta (Sec. "Parameter Efficient Finetuning (PEFT) Model Compression":
 * Theta_i = Theta_0 + lambda L_i, L_i = B A the adapter's dense update):
 *     L[r][c] = scale * sum_{t=0}^{rank-1} B[r][t] * A[t][c]
 * B is rows x rank, A is rank x cols, both row-major.  Accumulated in
 * binary64 (the reference value); abs_out, if not NULL, receives
 * |scale| * sum_t |B[r][t]| |A[t][c]|, which sizes the rounding bound of a
 * binary32 accumulation in any order.
 * ---------------------------------------------------------------------- */
void oracle_lora(const void *B, const void *A, int64_t rows, int64_t cols, int32_t rank,
                 double scale, int ab_dtype, double *out, double *abs_out)
{
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t c = 0; c < cols; ++c) {
            double acc = 0.0, mag = 0.0;
            for (int32_t t = 0; t < rank; ++t) {
                double b = (double)load_elem(B, r * rank + t, ab_dtype);
                double a = (double)load_elem(A, (int64_t)t * cols + c, ab_dtype);
                acc += b * a;
                mag += fabs(b) * fabs(a);
            }
            out[r * cols + c] = scale * acc;
            if (abs_out) abs_out[r * cols + c] = fabs(scale) * mag;
        }
    }
}

/* ------------------------------------------------------------------------
 * Superposition of LoRA adapters without materialising them (same section,
 * combined with Sec. 4.3 and Sec. 4.4):
 *     out[l][r][c] = scale * sum_i (-1)^{s(seed_i, l, c)} * sum_t B_i[src_i(l)][r][t] * A_i[src_i(l)][t][c]
 * in binary64.  Bs / As are indexed [i * n_layers + l] (original positions).
 * mag[l], if mag is not NULL, receives |scale| * sum_i sum_t |B||A|.
 * ---------------------------------------------------------------------- */
int oracle_lora_merge(const oracle_layer *layers, int32_t n_layers,
                      const void *const *Bs, const void *const *As, int32_t rank,
                      int32_t n_tasks, const uint64_t *seeds, double scale, int ab_dtype,
                      double *const *out, double *const *mag)
{
    int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers * (size_t)n_tasks);
    if (oracle_source_table(layers, n_layers, seeds, n_tasks, src) != 0) { free(src); return -1; }
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t m = layers[l].rows, n = layers[l].cols;
        uint8_t *sign = (uint8_t *)calloc((size_t)n * (size_t)n_tasks, 1);
        if (layers[l].flags & ORACLE_FLIP)
            for (int32_t i = 0; i < n_tasks; ++i)
                oracle_sign_mask(seeds[i], (uint32_t)l, n, sign + (int64_t)i * n);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < m; ++r) {
            for (int64_t c = 0; c < n; ++c) {
                double total = 0.0, total_mag = 0.0;
                for (int32_t i = 0; i < n_tasks; ++i) {
                    const int32_t t_layer = src[(int64_t)i * n_layers + l];
                    const void *B = Bs[(int64_t)i * n_layers + t_layer];
                    const void *A = As[(int64_t)i * n_layers + t_layer];
                    double acc = 0.0, am = 0.0;
                    for (int32_t t = 0; t < rank; ++t) {
                        double b = (double)load_elem(B, r * rank + t, ab_dtype);
                        double a = (double)load_elem(A, (int64_t)t * n + c, ab_dtype);
                        acc += b * a;
                        am += fabs(b) * fabs(a);
                    }
                    if (sign[(int64_t)i * n + c]) acc = -acc;
                    total += acc;
                    total_mag += am;
                }
                out[l][r * n + c] = scale * total;
                if (mag) mag[l][r * n + c] = fabs(scale) * total_mag;
            }
        }
        free(sign);
    }
    free(src);
    return 0;
}

/* ------------------------------------------------------------------------
 * Hot swap (Sec. "Model Hot Swapping"): add (sign = +1) or remove (sign = -1)
 * one model in place,
 *     Delta_*[l] <- Delta_*[l] + sign * (-1)^{s(seed, l, c)} * Delta_new[src(l)]
 * one binary32 addition per element on the stored superposition.
 * ---------------------------------------------------------------------- */
int oracle_update(const oracle_layer *layers, int32_t n_layers,
                  void *const *merged, int merged_dtype,
                  const void *const *delta, int delta_dtype,
                  uint64_t seed, int remove, int n_threads)
{
    int32_t *src = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers);
    if (oracle_source_table(layers, n_layers, &seed, 1, src) != 0) { free(src); return -1; }
#ifdef _OPENMP
    if (n_threads > 0) omp_set_num_threads(n_threads);
#endif
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t m = layers[l].rows, n = layers[l].cols;
        uint8_t *sign = (uint8_t *)calloc((size_t)n, 1);
        if (layers[l].flags & ORACLE_FLIP)
            oracle_sign_mask(seed, (uint32_t)l, n, sign);
#pragma omp parallel for schedule(static)
        for (int64_t r = 0; r < m; ++r) {
            for (int64_t c = 0; c < n; ++c) {
                float acc = load_elem(merged[l], r * n + c, merged_dtype);
                float x = load_elem(delta[src[l]], r * n + c, delta_dtype);
                if (sign[c]) x = -x;
                if (remove) x = -x;
                store_elem(merged[l], r * n + c, merged_dtype, acc + x);
            }
        }
        free(sign);
    }
    free(src);
    return 0;
}

/* ------------------------------------------------------------------------
 * Diagnostics of Sec. 3 ("Interference in Model Merging"): inner product and
 * squared norms of two equally long vectors in binary64, from which the
 * cosine similarity and the interference norm identity follow.
 * out3 = { <a,b>, <a,a>, <b,b> }.
 * ---------------------------------------------------------------------- */
void oracle_dot3(const void *a, const void *b, int64_t count, int dtype, double out3[3])
{
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int64_t e = 0; e < count; ++e) {
        double x = (double)load_elem(a, e, dtype), y = (double)load_elem(b, e, dtype);
        ab += x * y; aa += x * x; bb += y * y;
    }
    out3[0] = ab; out3[1] = aa; out3[2] = bb;
}

/* ------------------------------------------------------------------------
 * The same three sums for two transformed deltas over a whole stack:
 *     a'[l] = D_a^l-flipped a[src_a(l)],  b'[l] = D_b^l-flipped b[src_b(l)],
 * out3 = { <a',b'>, <a',a'>, <b',b'> } accumulated in binary64 in layer, row,
 * column order.  This is the "pairwise cosine similarity among interfering
 * deltas" of the experiments: the retrieving model's own D^-1 is orthogonal
 * and drops out of every inner product.
 * ---------------------------------------------------------------------- */
int oracle_delta_stats(const oracle_layer *layers, int32_t n_layers,
                       const void *const *a, uint64_t seed_a, const void *const *b, uint64_t seed_b,
                       int dtype, double out3[3])
{
    int32_t *sa = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers);
    int32_t *sb = (int32_t *)malloc(sizeof(int32_t) * (size_t)n_layers);
    if (oracle_source_table(layers, n_layers, &seed_a, 1, sa) != 0 ||
        oracle_source_table(layers, n_layers, &seed_b, 1, sb) != 0) { free(sa); free(sb); return -1; }
    double ab = 0.0, aa = 0.0, bb = 0.0;
    for (int32_t l = 0; l < n_layers; ++l) {
        const int64_t m = layers[l].rows, n = layers[l].cols;
        uint8_t *ma = (uint8_t *)calloc((size_t)n, 1), *mb = (uint8_t *)calloc((size_t)n, 1);
        if (layers[l].flags & ORACLE_FLIP) {
            oracle_sign_mask(seed_a, (uint32_t)l, n, ma);
            oracle_sign_mask(seed_b, (uint32_t)l, n, mb);
        }
        for (int64_t r = 0; r < m; ++r)
            for (int64_t c = 0; c < n; ++c) {
                double x = (double)load_elem(a[sa[l]], r * n + c, dtype);
                double y = (double)load_elem(b[sb[l]], r * n + c, dtype);
                if (ma[c]) x = -x;
                if (mb[c]) y = -y;
                ab += x * y; aa += x * x; bb += y * y;
            }
        free(ma); free(mb);
    }
    out3[0] = ab; out3[1] = aa; out3[2] = bb;
    free(sa); free(sb);
    return 0;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
