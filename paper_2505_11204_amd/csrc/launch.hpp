// Launchers of the gfx950 kernels, callable from plain C++ host code.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include "plan.hpp"

namespace randes {

constexpr int DT_F32 = 0, DT_BF16 = 1;

// vec = 0 launches the element-wise variant (one column per lane).
hipError_t launch_merge(const StreamArgs &a, int vec, int dt_in, int dt_out, hipStream_t s);
// Same with weights as inputs: srcs holds, per slot layer, T fine-tuned pointers then T base pointers.
hipError_t launch_merge_weights(const StreamArgs &a, int vec, int dt_in, int dt_out, hipStream_t s);
hipError_t launch_retrieve(const StreamArgs &a, int vec, int dt_merged, int dt_base, int dt_out, hipStream_t s);
hipError_t launch_update(const StreamArgs &a, int vec, int dt_merged, int dt_delta, hipStream_t s);
// a.n_tasks models (2, 4 or 8) retrieved in one pass; vector path only, one storage type.
hipError_t launch_retrieve_many(const StreamArgs &a, int dt, hipStream_t s);
// stats: per-workgroup partial triples into a.partials, then stats_finalize sums n_partials of them
// in a fixed order into out3 = { <a',b'>, <a',a'>, <b',b'> }.
hipError_t launch_stats(const StreamArgs &a, int vec, int dt, hipStream_t s);
hipError_t launch_stats_finalize(const double *partials, uint32_t n_partials, double *out3, hipStream_t s);
hipError_t launch_sign_mask(uint32_t key_lo, uint32_t key_hi, uint32_t layer, int64_t cols,
                            uint8_t *mask_out, hipStream_t s);

// One output matrix of a LoRA launch: out = scale * sum over its segments of B A D.
struct LoraItem {
    void *out;            // rows x cols
    int32_t rows, cols;
    uint32_t tiles_x;     // workgroup tiles along the columns
    uint32_t tile_begin;  // first workgroup of this matrix
    uint32_t seg_begin, n_seg;
};
// One term B A D of an output matrix.
struct LoraSeg {
    const void *B;        // rows x rank
    const void *A;        // rank x cols
    uint32_t key_lo, key_hi, layer_id, flip;   // the sign diagonal D (flip = 0: identity)
};
// Shape of a LoRA launch: nw waves side by side, nb blocks of 32 columns per wave (a workgroup's band
// is tile_cols = nw * nb * 32 columns wide); a workgroup walks down rb groups of rt blocks of 32 rows
// (32 * rt * rb rows per workgroup tile).
struct LoraShape { int nw, nb, rt, rb, tile_cols, res; };   // res: depth slices whose fragments of A stay in registers (0: streamed)
// The band width that wastes the fewest columns over the launch's matrices; rt from the depth of the
// deepest product (max_seg segments of `rank`); rb from the size of the launch.  Host code.
LoraShape lora_choose_shape(const LoraItem *items, size_t n_items, int32_t max_seg, int32_t rank, bool f32_factors, bool fast);
// wg_item_dev[t] = matrix of workgroup tile t (tiles of a matrix: column band fastest, then row block;
// tile_begin / tiles_x of the items computed for `shape`).  fast: every matrix has cols a multiple of 8,
// rank a multiple of 8 and 16-byte aligned operands; otherwise operands and results move by element.
hipError_t launch_lora(const LoraItem *items_dev, const LoraSeg *segs_dev, const uint32_t *wg_item_dev,
                       uint32_t n_tiles, const LoraShape &shape, bool fast, int32_t rank, float scale,
                       int dt_ab, int dt_out, hipStream_t s);

// Columns per lane of the vector kernels for a call whose widest-count stream
// holds bf16 (8) or only f32 (4).
int merge_vec(int dt_in);
int retrieve_vec(int dt_merged, int dt_base);
int update_vec(int dt_merged, int dt_delta);

// Rows of a tile one wave handles in its single load burst (the kernels' compile-time R).
int stats_vec(int dt);
int merge_burst_rows();
int merge_weights_burst_rows();
// Rows per wave of the kernel that retrieves q models in one pass: 4 * (1 + 8) = 36 or
// 8 * (1 + q) <= 40 sixteen-byte loads in flight per lane.
constexpr int retrieve_many_rows(int q) { return q >= 8 ? 4 : 8; }

// Two-input kernels (retrieve, update, stats): rows per burst so that about 32 sixteen-byte loads are
// in flight per lane: 16 rows when both streams fit 16 bytes per lane, fewer when a stream is wider.
// words_x / words_y = 32-bit words per lane and row of the two streams.
constexpr int two_input_rows(int words_x, int words_y)
{
    const int w = words_x + words_y;
    return w <= 8 ? 16 : (w <= 16 ? 8 : 4);
}
constexpr int stream_words(int dt, int vec) { return dt == DT_F32 ? vec : (vec == 1 ? 1 : vec / 2); }
inline int two_input_burst_rows(int dt_x, int dt_y, int vec)
{
    return two_input_rows(stream_words(dt_x, vec), stream_words(dt_y, vec));
}

// Plain streaming probe: out = sum of n_inputs streams (write != 0) or loads only (write == 0).
// bytes per stream must be a multiple of PROBE_CHUNK_BYTES.
constexpr uint64_t PROBE_CHUNK_BYTES = 4u * 256u * 16u;
hipError_t launch_probe(const void *const *inputs, int n_inputs, void *output, uint64_t bytes, int write, hipStream_t s);

constexpr int LORA_DEPTH_SLICE = 16;    // depth (segments x rank) values fetched and multiplied per step

}  // namespace randes
