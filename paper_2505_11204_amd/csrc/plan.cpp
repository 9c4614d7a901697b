// Host-side planning: argument checks, layer permutations and source tables,
// tile geometry.  Pure C++: nothing here needs a GPU.
#include "plan.hpp"

#include <algorithm>
#include <map>
#include <numeric>

#include "philox.hpp"

namespace randes {

// sigma ~ S_G (Sec. 4.3): every position draws a 64-bit key from the generator;
// sigma is the stable ascending argsort of the keys.
void layer_perm(uint64_t seed, int32_t group, int32_t group_size, int32_t *perm_out)
{
    const uint32_t klo = (uint32_t)(seed & 0xffffffffu), khi = (uint32_t)(seed >> 32);
    std::vector<uint64_t> keys((size_t)group_size);
    for (int32_t k = 0; k < group_size; ++k) {
        const u32x4_t o = philox4x32_10((uint32_t)k, (uint32_t)group, STREAM_PERM, 0u, klo, khi);
        keys[(size_t)k] = ((uint64_t)o.w[0] << 32) | (uint64_t)o.w[1];
    }
    std::iota(perm_out, perm_out + group_size, 0);
    std::stable_sort(perm_out, perm_out + group_size,
                     [&](int32_t a, int32_t b) { return keys[(size_t)a] < keys[(size_t)b]; });
}

int validate_layers(const randes_layer *layers, int32_t n_layers, std::string *why)
{
    if (!layers || n_layers < 1) { *why = "layers is NULL or n_layers < 1"; return RANDES_EINVAL; }
    for (int32_t l = 0; l < n_layers; ++l) {
        if (layers[l].rows < 1 || layers[l].cols < 1) { *why = "layer with rows < 1 or cols < 1"; return RANDES_EINVAL; }
        if (layers[l].cols >= (int64_t)1 << 31 || layers[l].rows >= (int64_t)1 << 31) {
            *why = "layer with rows or cols >= 2^31"; return RANDES_ENOTSUP;
        }
        if (layers[l].flags & ~(RANDES_FLIP | RANDES_SHUFFLE | RANDES_SHIFT)) { *why = "unknown layer flag"; return RANDES_EINVAL; }
    }
    return RANDES_OK;
}

static bool movable(const randes_layer &l) { return l.group >= 0 && (l.flags & (RANDES_SHUFFLE | RANDES_SHIFT)); }

int build_source_table(const randes_layer *layers, int32_t n_layers, uint64_t seed,
                       std::vector<int32_t> *src, std::string *why)
{
    src->resize((size_t)n_layers);
    std::iota(src->begin(), src->end(), 0);
    std::map<int32_t, std::vector<int32_t>> groups;   // group id -> member layers, ascending
    for (int32_t l = 0; l < n_layers; ++l)
        if (movable(layers[l])) groups[layers[l].group].push_back(l);
    std::vector<int32_t> perm;
    for (const auto &kv : groups) {
        const std::vector<int32_t> &mem = kv.second;
        const int32_t G = (int32_t)mem.size();
        bool shift = false;
        for (int32_t l : mem) {
            if (layers[l].rows != layers[mem[0]].rows || layers[l].cols != layers[mem[0]].cols) {
                *why = "layers of one shuffle group differ in shape"; return RANDES_EINVAL;
            }
            shift = shift || (layers[l].flags & RANDES_SHIFT);
        }
        perm.resize((size_t)G);
        if (shift) {
            // layer shifting: the whole group moves `dist` slots deeper, cyclically.  The distance is
            // the model's own (one more than its seed, modulo the group size), so that two models are
            // shifted against each other and not merely relabelled together.
            const int32_t dist = (int32_t)((seed % (uint64_t)G + 1u) % (uint64_t)G);
            for (int32_t k = 0; k < G; ++k) perm[(size_t)k] = (k + G - dist) % G;   // slot k receives layer k - dist
        } else {
            layer_perm(seed, kv.first, G, perm.data());
        }
        for (int32_t k = 0; k < G; ++k) (*src)[(size_t)mem[(size_t)k]] = mem[(size_t)perm[(size_t)k]];
    }
    return RANDES_OK;
}

// Idle share of the lanes for rows of `cols` columns under the best of the allowed tile widths.
static double idle_share(uint64_t cols, int vec, int max_wx_shift)
{
    double best = 1.0;
    for (int sh = 0; sh <= max_wx_shift; ++sh) {
        const uint64_t cw = (uint64_t)(64 * vec) << sh;
        const uint64_t span = (cols + cw - 1) / cw * cw;
        best = std::min(best, (double)(span - cols) / (double)span);
    }
    return best;
}

int fold_factor(int64_t rows, int64_t cols, int vec, int max_wx_shift)
{
    if (cols % 128 != 0 || cols % vec != 0) return 1;
    const double plain = idle_share((uint64_t)cols, vec, max_wx_shift);
    if (plain <= 0.05) return 1;   // 11008 bf16 columns idle 2.3 % of the lanes: folding them measured 1 % slower
    int best_f = 1;
    double best = plain;
    for (int f = 2; f <= 8; ++f) {
        if (rows < f || (int64_t)f * cols >= ((int64_t)1 << 31)) break;
        const double idle = idle_share((uint64_t)f * (uint64_t)cols, vec, max_wx_shift);
        if (idle < best - 0.01) { best = idle; best_f = f; }   // a longer fold must earn its remainder rows
    }
    return best_f;
}

uint64_t plan_layer_geometry(LayerDev *d, int vec, int rows_per_wave, int max_wx_shift)
{
    const uint64_t cols = (uint64_t)d->cols, rows = (uint64_t)d->rows;
    // waves along the columns: the arrangement that wastes the fewest lanes; among equals the
    // narrowest (4 waves stacked along the rows measured 1-2 % faster than 4 side by side on rows of
    // 8 KB), except on rows of 20 KB and more, where the widest of the equals is faster (11008 bf16
    // columns with 2 waves side by side instead of 1: retrieve +0.5 %, merge +0.2 % on the 7B shapes)
    const bool long_rows = vec > 1 && cols / (uint64_t)vec * 16u >= LONG_ROW_BYTES;
    uint32_t best_shift = 0;
    uint64_t best_waste = ~0ull;
    for (int sh = 0; sh <= max_wx_shift; ++sh) {
        const uint64_t cw = (uint64_t)(64 * vec) << sh;
        const uint64_t waste = (cols + cw - 1) / cw * cw - cols;
        if (waste < best_waste || (long_rows && waste == best_waste)) { best_waste = waste; best_shift = (uint32_t)sh; }
    }
    d->wx_shift = best_shift;
    d->wx = 1u << best_shift;
    const uint64_t cw = (uint64_t)(64 * vec) << best_shift;
    d->n_cb = (uint32_t)((cols + cw - 1) / cw);
    // in-tile byte offsets are 32-bit: tile_rows * cols * 4 (the widest element) must stay below 2^32
    const uint64_t row_bytes = cols * 4;
    const uint64_t max_rows = (((uint64_t)1 << 32) - 1) / row_bytes;
    if (max_rows < 1) return 0;
    uint64_t tr = (uint64_t)rows_per_wave << (2 - best_shift);   // 4 waves: 4 / wx of them stacked along the rows
    if (tr > max_rows) tr = max_rows;
    if (tr > rows) tr = rows;
    if (tr < 1) tr = 1;
    d->tile_rows = (uint32_t)tr;
    const uint64_t n_rc = (rows + tr - 1) / tr;
    return n_rc * d->n_cb;
}

void build_coarse_index(SubPlan *sp)
{
    sp->coarse.clear();
    if (sp->layers.empty()) { sp->coarse.assign(2, 0u); return; }
    const uint32_t n_chunks = (sp->n_tiles + 1023u) / 1024u;
    uint32_t layer = 0;
    for (uint32_t i = 0; i <= n_chunks; ++i) {
        const uint64_t tile = std::min<uint64_t>((uint64_t)i * 1024u, sp->n_tiles ? sp->n_tiles - 1u : 0u);
        while (layer + 1 < sp->layers.size() && sp->tile_begin[layer + 1] <= tile) ++layer;
        sp->coarse.push_back(layer);
    }
}

int two_input_default_rows(int burst, double stream_bytes)
{
    double share = stream_bytes / 3.2e9;
    share = share < 0.375 ? 0.375 : (share > 0.75 ? 0.75 : share);
    const int rows = (int)(burst * share + 0.5);
    return rows < 1 ? 1 : rows;
}

uint32_t wide_row_lds_floor(const SubPlan &sub, size_t elem_bytes)
{
    // the length of the row an average byte of the launch lies in; rows as the kernels see them
    // (folded layers: the longer row)
    double bytes = 0.0, weighted = 0.0;
    for (const LayerDev &d : sub.layers) {
        const double row = (double)d.cols * (double)elem_bytes, b = (double)d.rows * row;
        bytes += b;
        weighted += b * row;
    }
    return bytes > 0.0 && weighted / bytes >= (double)WIDE_ROW_BYTES ? TWO_WORKGROUP_LDS : 0u;
}

}  // namespace randes
