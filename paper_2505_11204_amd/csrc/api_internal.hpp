// Host-side pieces shared by the translation units that implement the C ABI: error text, launch-shape
// knobs, turning a host plan into one table image, and the plan builders that more than one entry
// point uses.  Nothing here touches the device.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "plan.hpp"

namespace randes {

// Record the text of a failure for randes_strerror() on this thread and hand the code back.
int fail(int code, const std::string &why);
int hip_fail(hipError_t e, const char *what);

inline bool dtype_ok(int d) { return d == RANDES_F32 || d == RANDES_BF16; }
inline size_t elem_bytes(int d) { return d == RANDES_F32 ? 4 : 2; }
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
inline bool elem_aligned(const void *p, int dtype) { return ((uintptr_t)p & (elem_bytes(dtype) - 1)) == 0; }

// Launch-shape knobs of the calling thread (measurement aids; results never depend on them).
struct Knobs {
    int merge_rows = 0, retrieve_rows = 0;   // rows per wave per tile; 0 = the kernels' burst size
    int max_wx_shift = 2;                    // widest tile: 4 waves side by side along the columns
    int fold = 1;                            // rows of layers that leave lanes idle are folded
    int32_t word(int rows) const { return rows * 16 + max_wx_shift * 2 + fold; }   // for cache keys
};
Knobs &knobs();

// Where the tables of a host plan lie inside its one image (byte offsets, 256-byte aligned).
struct TableLayout {
    size_t layers[2], srcs[2], tile_begin[2], coarse[2];   // [0] vector sub-plan, [1] element-wise
    size_t keys, extra, total;
};

// Serialise a host plan (builds its coarse indices first).  `image` receives `total` bytes; the
// `extra` region (scratch of hp.extra_bytes) is left zero and lies last.
void pack_tables(HostPlan &hp, std::vector<char> *image, TableLayout *lay);

// Kernel arguments that point into an image resident at device address `dev_base`.
void bind_tables(const void *dev_base, const TableLayout &lay, const HostPlan &hp, int n_tasks,
                 StreamArgs *vec, StreamArgs *scl);

// Sec. 3 diagnostics (randes_delta_stats): argument checks, and the plan of a call whose arguments
// passed them (descriptors of both transformed deltas per slot layer; hp->extra_bytes = room for one
// triple of partial sums per workgroup).
int validate_stats_args(const randes_layer *layers, int32_t n_layers,
                        const void *const *delta_a, const void *const *delta_b, int dtype, const double *out3);
int build_stats_plan(const randes_layer *layers, int32_t n_layers,
                     const void *const *delta_a, uint64_t seed_a,
                     const void *const *delta_b, uint64_t seed_b,
                     int dtype, HostPlan *hp);

}  // namespace randes
