// Host-side plan of one merge / retrieve / update call and the device-resident
// tables the streaming kernels read.  A plan turns the caller's layer list and
// pointer arrays into: the per-model source tables (Sec. 4.3: the shuffle is a
// pointer reallocation), per-layer descriptors, and a tile decomposition.
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/randes.h"

namespace randes {

// One slot layer as a kernel sees it.  Pointers are device pointers.
struct LayerDev {
    void *dst;          // merge/update: merged[l];  retrieve: out[src(l)]
    const void *a;      // retrieve: merged[l];      update: delta[src(l)]
    const void *b;      // retrieve: base[src(l)]
    int32_t rows;
    int32_t cols;
    uint32_t layer_id;  // slot index l: the generator's layer coordinate
    uint32_t flip;      // 1 if the layer takes the sign flip
    uint32_t n_cb;      // column blocks per row chunk
    uint32_t tile_rows; // rows per tile
    uint32_t wx;        // waves of a workgroup laid along the columns (1, 2 or 4)
    uint32_t wx_shift;  // log2(wx)
    uint32_t sign_blocks;  // 0, or: this descriptor shows several rows of the layer as one (rows folded),
                           // and the sign pattern repeats every sign_blocks generator blocks of 128 columns
};

// What a streaming kernel receives by value.
struct StreamArgs {
    const LayerDev *layers;       // n_layers
    const void *const *srcs;      // merge: [n_layers][n_tasks] source pointers (several retrievals: base, then output pointers)
    const uint32_t *tile_begin;   // n_layers + 1 prefix sums of tiles
    const uint32_t *coarse;       // coarse[i] = layer that holds tile 1024 * i (one extra entry at the end)
    const uint32_t *keys;         // merge only: [n_tasks][2] = (seed low, seed high)
    int32_t n_layers;
    int32_t n_tasks;
    uint32_t n_tiles;
    uint32_t key_lo, key_hi;      // retrieve / update: the one model's seed
    float lambda;                 // retrieve
    float lambdas[8];             // several retrievals in one pass: one scale per model
    uint32_t negate;              // update: 1 removes the model
    uint32_t key2_lo, key2_hi;    // stats: the second model's seed
    double *partials;             // stats: one triple per workgroup
    uint32_t partial_base;        // stats: index of this launch's first triple
    uint32_t lds_floor;           // dynamic LDS to request at least (bytes; 0 = what the kernel needs): see wide_row_lds_floor()
    uint32_t xcd_chunk_shift;     // how the tile sequence is dealt to the 8 XCDs: 0 = one contiguous eighth each,
                                  // s > 0 = chunks of 1 << s tiles in turn (see locate() in kernels.hip)
};

// Two workgroups per CU instead of three.  Measured on MI355X: retrieve, hot swap and the merge of 3
// to 8 tasks held in registers stream 1-3 % faster with two workgroups (8 waves) per CU than with the
// three or four their registers allow, on stacks of long rows (with 2 tasks too little is in flight
// then: -8 %); on stacks of short rows (T5-base: 1.5 to 4 KB)
// and for the kernels that keep fewer bytes in flight per wave (the any-count merge, the read-only
// diagnostics) more workgroups are better.  Occupancy is set per launch by the size of the LDS
// request: 80 KB of the CU's 160 KB leave room for two workgroups.
constexpr uint32_t WIDE_ROW_BYTES = 6144;       // row length, averaged over the launch's bytes, from which the launch is capped
constexpr uint32_t TWO_WORKGROUP_LDS = 81920;
// The merge of deltas deals its tiles to the XCDs in chunks of 32 instead of one contiguous eighth each
// when it reads less than 80 GB: measured on MI355X, T5-base +4.7 %, ViT-B/32 +3.6 %, ViT-L/14 +1.2 %,
// 8 to 24 Llama blocks +1 % (with ordinary allocations 3.6 to 5 % on the three small stacks); from 29 blocks
// (94 GB) on the contiguous order is 0.4-0.5 % faster.  Retrieve is slower with chunks at every size.
constexpr uint32_t MERGE_CHUNK_SHIFT = 5;
constexpr double MERGE_CHUNKED_BELOW_BYTES = 80e9;
constexpr uint64_t LONG_ROW_BYTES = 20480;      // row length from which a layer's tiles are as wide as they can be without idling more lanes
struct SubPlan;
uint32_t wide_row_lds_floor(const SubPlan &sub, size_t elem_bytes);

// Rows a wave of retrieve or hot swap takes of its tile when the caller has not set the knob: a share
// of the kernel's burst of `burst` rows that grows with the bytes of the stream the flip acts on.
// A workgroup lives about as long as the memory takes to serve what all resident workgroups have
// asked for (15 us with full bursts), and at the end of a launch the last ones finish one by one
// over that time, so a stack the chip streams in a few hundred microseconds wants short-lived
// workgroups: 3/8 of the burst up to 1.2 GB.  Long launches take 3/4 of it (from 2.4 GB): measured
// on MI355X, two workgroups per CU with 12 rows a wave, or three with 8, stream 0.4 % faster than
// two with 16, and fewer rows in flight than that lose again.  Hot swap works in place and takes
// the short burst at every size (it passes 0 bytes).
int two_input_default_rows(int burst, double stream_bytes);


// A sub-plan: the layers one kernel variant handles (vector or element-wise).
struct SubPlan {
    std::vector<LayerDev> layers;
    std::vector<const void *> srcs;     // merge
    std::vector<uint32_t> tile_begin;
    std::vector<uint32_t> coarse;
    uint32_t n_tiles = 0;
};

struct HostPlan {
    SubPlan vec, scl;
    std::vector<uint32_t> keys;
    size_t extra_bytes = 0;   // scratch appended to the device tables (stats: per-workgroup partials)
};

enum PlanKind { PLAN_MERGE = 1, PLAN_RETRIEVE = 2, PLAN_UPDATE = 3, PLAN_MERGE_WEIGHTS = 4, PLAN_STATS = 5,
                PLAN_RETRIEVE_MANY = 6, PLAN_LORA = 7, PLAN_LORA_MERGE = 8 };

int validate_layers(const randes_layer *layers, int32_t n_layers, std::string *why);

// src[l] = layer of this model that lands in slot l.
int build_source_table(const randes_layer *layers, int32_t n_layers, uint64_t seed,
                       std::vector<int32_t> *src, std::string *why);

void layer_perm(uint64_t seed, int32_t group, int32_t group_size, int32_t *perm_out);

// Fill the geometry (n_cb, wx, tile_rows) of one descriptor for lanes that own
// `vec` columns each and waves that own `rows_per_wave` rows of a tile; returns
// the layer's tile count, or 0 if the layer is too wide for 32-bit in-tile offsets.
uint64_t plan_layer_geometry(LayerDev *d, int vec, int rows_per_wave, int max_wx_shift = 2);

// How many consecutive rows of a rows x cols layer to show to the kernels as one row, so that fewer
// lanes of the 64 * vec * {1, 2, 4} column wide tiles hang over the end of a row (768 bf16 columns
// leave a quarter of the lanes idle; two rows = 1536 columns leave none).  1 = leave the layer as it
// is.  Folding needs cols to be a multiple of 128, the generator's block, so that a block of the
// folded row is a whole block of the sign pattern.
int fold_factor(int64_t rows, int64_t cols, int vec, int max_wx_shift = 2);

// coarse[i] = layer holding tile 1024 * i, for i = 0 .. ceil(n_tiles / 1024).
void build_coarse_index(SubPlan *sp);

}  // namespace randes
