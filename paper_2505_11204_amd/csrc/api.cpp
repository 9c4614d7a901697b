// C ABI of the library (see include/randes.h): argument validation, plan cache,
// table upload and kernel launches.  No arithmetic of the method happens on the
// host except the layer permutations, which are pointer bookkeeping (Sec. 4.3).
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <list>
#include <memory>
#include <mutex>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/randes_bench.h"
#include "api_internal.hpp"
#include "launch.hpp"
#include "plan.hpp"

using namespace randes;

namespace randes {

namespace {
thread_local std::string g_detail;   // text of the last failure on this thread
thread_local Knobs g_knobs;          // launch-shape knobs of this thread
}  // namespace

int fail(int code, const std::string &why)
{
    g_detail = why;
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    g_detail = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();   // clear the sticky error so the next call starts clean
    return RANDES_EHIP;
}

Knobs &knobs() { return g_knobs; }

void pack_tables(HostPlan &hp, std::vector<char> *image, TableLayout *lay)
{
    auto pad = [](size_t x) { return (x + 255) & ~(size_t)255; };
    build_coarse_index(&hp.vec);
    build_coarse_index(&hp.scl);
    const SubPlan *sub[2] = { &hp.vec, &hp.scl };
    size_t off = 0;
    for (int s = 0; s < 2; ++s) {
        lay->layers[s] = off;     off = pad(off + sub[s]->layers.size() * sizeof(LayerDev));
        lay->srcs[s] = off;       off = pad(off + sub[s]->srcs.size() * sizeof(void *));
        lay->tile_begin[s] = off; off = pad(off + sub[s]->tile_begin.size() * sizeof(uint32_t));
        lay->coarse[s] = off;     off = pad(off + sub[s]->coarse.size() * sizeof(uint32_t));
    }
    lay->keys = off;
    off = pad(off + hp.keys.size() * sizeof(uint32_t));
    lay->extra = off;   // last, so that an image can be shipped without its scratch
    off = pad(off + hp.extra_bytes);
    lay->total = off;
    image->assign(lay->extra, 0);
    char *host = image->data();
    for (int s = 0; s < 2; ++s) {
        if (!sub[s]->layers.empty()) memcpy(host + lay->layers[s], sub[s]->layers.data(), sub[s]->layers.size() * sizeof(LayerDev));
        if (!sub[s]->srcs.empty()) memcpy(host + lay->srcs[s], sub[s]->srcs.data(), sub[s]->srcs.size() * sizeof(void *));
        if (!sub[s]->tile_begin.empty()) memcpy(host + lay->tile_begin[s], sub[s]->tile_begin.data(), sub[s]->tile_begin.size() * sizeof(uint32_t));
        memcpy(host + lay->coarse[s], sub[s]->coarse.data(), sub[s]->coarse.size() * sizeof(uint32_t));
    }
    if (!hp.keys.empty()) memcpy(host + lay->keys, hp.keys.data(), hp.keys.size() * sizeof(uint32_t));
}

void bind_tables(const void *dev_base, const TableLayout &lay, const HostPlan &hp, int n_tasks,
                 StreamArgs *vec, StreamArgs *scl)
{
    const SubPlan *sub[2] = { &hp.vec, &hp.scl };
    StreamArgs *args[2] = { vec, scl };
    const char *b = (const char *)dev_base;
    for (int s = 0; s < 2; ++s) {
        StreamArgs &a = *args[s];
        memset(&a, 0, sizeof(a));
        a.layers = (const LayerDev *)(b + lay.layers[s]);
        a.srcs = (const void *const *)(b + lay.srcs[s]);
        a.tile_begin = (const uint32_t *)(b + lay.tile_begin[s]);
        a.coarse = (const uint32_t *)(b + lay.coarse[s]);
        a.keys = (const uint32_t *)(b + lay.keys);
        a.n_layers = (int32_t)sub[s]->layers.size();
        a.n_tasks = n_tasks;
        a.n_tiles = sub[s]->n_tiles;
    }
}

}  // namespace randes

namespace {

// A wave handles one burst of at most `burst` rows; the knob can only shrink it.
int clamp_rows(int knob, int burst) { return (knob <= 0 || knob > burst) ? burst : knob; }

// The same for retrieve and hot swap, whose default depends on the size of the stack.
// (Element-wise layers keep the full burst: their lanes hold 2 or 4 bytes a row, not 16.)
int two_input_rows_for(int knob, int burst, double stream_bytes, bool vector_ok)
{
    return (knob > 0 || !vector_ok) ? clamp_rows(knob, burst) : two_input_default_rows(burst, stream_bytes);
}

double stack_bytes(const randes_layer *layers, int32_t n_layers, int dtype)
{
    double b = 0.0;
    for (int32_t l = 0; l < n_layers; ++l) b += (double)layers[l].rows * (double)layers[l].cols * (double)elem_bytes(dtype);
    return b;
}

// ------------------------------------------------------------------ plan cache
// A call's device tables are found by what the call was given: the kind of call, the layer list,
// every pointer and seed.  The arguments are hashed where they lie (no copy on the cached path) and
// compared piece by piece on a hash match; the copy is made once, when the tables are built.
struct CallKey {
    struct Piece { const void *p; size_t n; };
    Piece piece[10];
    int n_pieces = 0;
    void add(const void *p, size_t n) { piece[n_pieces++] = Piece{ p, n }; }
    uint64_t hash() const
    {
        uint64_t h = 0x243f6a8885a308d3ull;
        for (int q = 0; q < n_pieces; ++q) {
            const unsigned char *b = (const unsigned char *)piece[q].p;
            size_t n = piece[q].n;
            h = (h ^ (uint64_t)n) * 0x9e3779b97f4a7c15ull;
            for (; n >= 8; n -= 8, b += 8) {
                uint64_t w;
                memcpy(&w, b, 8);
                h = (h ^ w) * 0x9e3779b97f4a7c15ull;
                h ^= h >> 29;
            }
            uint64_t w = 0;
            if (n) memcpy(&w, b, n);
            h = (h ^ w) * 0x9e3779b97f4a7c15ull;
            h ^= h >> 32;
        }
        return h;
    }
    size_t bytes() const { size_t t = 0; for (int q = 0; q < n_pieces; ++q) t += piece[q].n; return t; }
    bool equals(const std::string &stored) const
    {
        if (stored.size() != bytes()) return false;
        size_t off = 0;
        for (int q = 0; q < n_pieces; ++q) {
            if (memcmp(stored.data() + off, piece[q].p, piece[q].n) != 0) return false;
            off += piece[q].n;
        }
        return true;
    }
    std::string str() const
    {
        std::string s;
        s.reserve(bytes());
        for (int q = 0; q < n_pieces; ++q) s.append((const char *)piece[q].p, piece[q].n);
        return s;
    }
};

struct CachedPlan {
    std::string key;
    uint64_t hash = 0;
    int device = 0;
    void *blob = nullptr;     // device tables
    size_t blob_bytes = 0;
    void *extra = nullptr;    // scratch inside the blob (stats partials)
    bool pinned = false;      // recorded into a HIP graph: its tables must outlive the cache's turnover
    StreamArgs vec{}, scl{};
    // LoRA launches: where the segment and workgroup tables start, and the launch shape chosen for them
    size_t items_bytes = 0, segs_bytes = 0;
    uint32_t lora_tiles = 0;
    LoraShape lora_shape{};
    bool lora_fast = false;
};
using PlanRef = std::shared_ptr<CachedPlan>;

// g_mu guards the three containers below and the `pinned` flags, for the length of a lookup or
// an insertion only: host planning, uploads and kernel launches all happen outside it.
std::mutex g_mu;
std::list<PlanRef> g_lru;                                                       // most recently used first
std::unordered_multimap<uint64_t, std::list<PlanRef>::iterator> g_index;        // by hash of the call
// Argument sets dropped from the cache.  Their tables are not freed at once (kernels already enqueued
// may still read them, and a caller may hold a set it looked up a moment ago): they wait here and
// are released in batches by reclaim_retired(), the rest by randes_shutdown().
std::vector<PlanRef> g_retired;
size_t g_retired_bytes = 0;
constexpr size_t RETIRED_LIMIT = (size_t)64 << 20;   // retired table bytes that trigger a release
size_t g_pinned = 0;
constexpr size_t MAX_PLANS = 256;     // argument sets kept (beyond those recorded into graphs)
constexpr size_t MAX_PINNED = 4096;   // argument sets recorded into graphs

PlanRef lookup_locked(uint64_t h, const CallKey &k, int device)
{
    auto range = g_index.equal_range(h);
    for (auto it = range.first; it != range.second; ++it) {
        const PlanRef &p = *it->second;
        if (p->device == device && k.equals(p->key)) {
            g_lru.splice(g_lru.begin(), g_lru, it->second);
            return p;
        }
    }
    return nullptr;
}

void insert_locked(const PlanRef &p)
{
    g_lru.push_front(p);
    g_index.emplace(p->hash, g_lru.begin());
    // Drop the least recently used argument sets beyond the limit, never those a graph refers to.
    // Their tables are not freed here (hipFree waits for the whole device and is not allowed while
    // a stream is being captured; kernels already enqueued may still read them): they are retired.
    size_t loose = g_lru.size() - g_pinned;
    for (auto it = g_lru.end(); loose > MAX_PLANS && it != g_lru.begin();) {
        --it;
        if ((*it)->pinned || it == g_lru.begin()) continue;
        auto range = g_index.equal_range((*it)->hash);
        for (auto ix = range.first; ix != range.second; ++ix)
            if (ix->second == it) { g_index.erase(ix); break; }
        if ((*it)->blob) { g_retired_bytes += (*it)->blob_bytes; g_retired.push_back(*it); }
        it = g_lru.erase(it);
        --loose;
    }
}

// Release the retired tables of this device once they add up to RETIRED_LIMIT, so that a loop that
// cycles over more argument sets than the cache keeps does not grow device memory without bound.
// Only sets nobody else holds are taken (a holder could still launch with them), and everything
// launched before is drained first.  Called from the path that has just allocated and copied
// synchronously itself (a first call, never under capture), never with g_mu held.
void reclaim_retired(int dev)
{
    std::vector<PlanRef> victims;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (g_retired_bytes <= RETIRED_LIMIT) return;
        std::vector<PlanRef> keep;
        for (PlanRef &p : g_retired) {
            if (p->device == dev && p.use_count() == 1) { g_retired_bytes -= p->blob_bytes; victims.push_back(std::move(p)); }
            else keep.push_back(std::move(p));
        }
        g_retired.swap(keep);
    }
    if (victims.empty()) return;
    if (hipDeviceSynchronize() != hipSuccess) {   // not now (e.g. a capture elsewhere forbids it): keep them
        (void)hipGetLastError();
        std::lock_guard<std::mutex> lock(g_mu);
        for (PlanRef &p : victims) { g_retired_bytes += p->blob_bytes; g_retired.push_back(std::move(p)); }
        return;
    }
    for (PlanRef &p : victims) {
        (void)hipFree(p->blob);
        p->blob = nullptr;
    }
}

bool stream_is_capturing(void *hip_stream)
{
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing((hipStream_t)hip_stream, &st) == hipSuccess) return st == hipStreamCaptureStatusActive;
    (void)hipGetLastError();
    return false;
}

int current_device(int *dev)
{
    hipError_t e = hipGetDevice(dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    return RANDES_OK;
}

// The tables of the call described by `k`: cached, or built now by `build(CachedPlan *)`, which
// plans on the host and uploads (and leaves no allocation behind when it fails).  A call recorded
// into a graph is replayed with kernel arguments that point into its tables, so those are kept
// until randes_shutdown(); the first call with an argument set allocates and copies synchronously
// and is therefore refused while its stream is being captured.
template <class Build, class Precheck>
int find_or_build(const CallKey &k, void *hip_stream, PlanRef *out, Build build, Precheck precheck);
template <class Build>
int find_or_build(const CallKey &k, void *hip_stream, PlanRef *out, Build build)
{
    return find_or_build(k, hip_stream, out, build, []() { return (int)RANDES_OK; });
}

// `precheck` holds argument checks that are too costly for every call and whose verdict is the same
// for equal arguments (overlap sweeps): it runs when the argument set is not cached, before
// anything else, and also when no device can be asked, so that a bad argument is reported as such
// on any machine.
template <class Build, class Precheck>
int find_or_build(const CallKey &k, void *hip_stream, PlanRef *out, Build build, Precheck precheck)
{
    int dev, rc;
    if ((rc = current_device(&dev))) {
        const std::string no_device = randes_strerror(rc);
        if (int bad = precheck()) return bad;
        return fail(rc, no_device);
    }
    const uint64_t h = k.hash();
    const bool capturing = stream_is_capturing(hip_stream);
    {
        std::lock_guard<std::mutex> lock(g_mu);
        PlanRef p = lookup_locked(h, k, dev);
        if (p) {
            if (capturing && !p->pinned) {
                if (g_pinned >= MAX_PINNED)
                    return fail(RANDES_ENOTSUP, "too many argument sets recorded into graphs; randes_shutdown() releases them");
                p->pinned = true;
                ++g_pinned;
            }
            *out = p;
            return RANDES_OK;
        }
    }
    if (int bad = precheck()) return bad;
    if (capturing)
        return fail(RANDES_ENOTSUP, "the first call with an argument set uploads its tables and cannot be recorded: "
                                    "call once eagerly before capturing the stream");
    PlanRef fresh = std::make_shared<CachedPlan>();
    fresh->key = k.str();
    fresh->hash = h;
    fresh->device = dev;
    if ((rc = build(fresh.get()))) return rc;
    std::unique_lock<std::mutex> lock(g_mu);
    PlanRef p = lookup_locked(h, k, dev);
    if (p) {   // another thread built the same tables meanwhile: use those
        if (fresh->blob) { g_retired_bytes += fresh->blob_bytes; g_retired.push_back(fresh); }
        *out = p;
        return RANDES_OK;
    }
    insert_locked(fresh);
    *out = fresh;
    const bool full = g_retired_bytes > RETIRED_LIMIT;
    lock.unlock();
    if (full) reclaim_retired(dev);
    return RANDES_OK;
}

// Lay the host plan out in one blob, upload it, and fill the kernel arguments.
int upload(HostPlan &hp, int n_tasks, CachedPlan *cp)
{
    std::vector<char> image;
    TableLayout lay;
    pack_tables(hp, &image, &lay);
    hipError_t e = hipMalloc(&cp->blob, lay.total);
    if (e != hipSuccess) { cp->blob = nullptr; return hip_fail(e, "hipMalloc(plan tables)"); }
    cp->blob_bytes = lay.total;
    e = hipMemcpy(cp->blob, image.data(), image.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(cp->blob); cp->blob = nullptr; return hip_fail(e, "hipMemcpy(plan tables)"); }
    cp->extra = hp.extra_bytes ? (char *)cp->blob + lay.extra : nullptr;
    bind_tables(cp->blob, lay, hp, n_tasks, &cp->vec, &cp->scl);
    return RANDES_OK;
}

// Bytes per element of the streams a descriptor points to (for pointer arithmetic on pieces of a layer).
struct StreamBytes { size_t dst, a, b, src; };

int place_piece(HostPlan *hp, LayerDev d, const void *const *srcs, int n_srcs, bool vector_ok, int vec, int rows_per_wave);

// Add one slot layer to the vector or element-wise sub-plan.  A layer on the vector path whose row
// length leaves lanes idle goes in folded: f rows shown as one, plus the rows % f rows left over.
int place(HostPlan *hp, LayerDev d, const void *const *srcs, int n_srcs, bool vector_ok, int vec, int rows_per_wave,
          const StreamBytes &eb)
{
    const Knobs &kn = knobs();
    const int f = (vector_ok && kn.fold) ? fold_factor(d.rows, d.cols, vec, kn.max_wx_shift) : 1;
    if (f <= 1) return place_piece(hp, d, srcs, n_srcs, vector_ok, vec, rows_per_wave);
    const int64_t rows = d.rows, cols = d.cols;
    LayerDev fd = d;
    fd.rows = (int32_t)(rows / f);
    fd.cols = (int32_t)(cols * f);
    fd.sign_blocks = (uint32_t)(cols / 128);
    int rc = place_piece(hp, fd, srcs, n_srcs, true, vec, rows_per_wave);
    if (rc || rows % f == 0) return rc;
    const size_t skip = (size_t)(rows / f) * (size_t)f * (size_t)cols;   // elements before the left-over rows
    LayerDev rd = d;
    rd.rows = (int32_t)(rows % f);
    if (rd.dst) rd.dst = (char *)rd.dst + skip * eb.dst;
    if (rd.a) rd.a = (const char *)rd.a + skip * eb.a;
    if (rd.b) rd.b = (const char *)rd.b + skip * eb.b;
    std::vector<const void *> moved((size_t)n_srcs);
    for (int i = 0; i < n_srcs; ++i) moved[(size_t)i] = (const char *)srcs[i] + skip * eb.src;
    return place_piece(hp, rd, moved.data(), n_srcs, true, vec, rows_per_wave);
}

int place_piece(HostPlan *hp, LayerDev d, const void *const *srcs, int n_srcs, bool vector_ok, int vec, int rows_per_wave)
{
    SubPlan &sp = vector_ok ? hp->vec : hp->scl;
    const uint64_t tiles = plan_layer_geometry(&d, vector_ok ? vec : 1, rows_per_wave, knobs().max_wx_shift);
    if (tiles == 0) return fail(RANDES_ENOTSUP, "layer too wide for 32-bit in-tile offsets");
    if ((uint64_t)sp.n_tiles + tiles >= ((uint64_t)1 << 31)) return fail(RANDES_ENOTSUP, "too many tiles for one launch");
    if (sp.tile_begin.empty()) sp.tile_begin.push_back(0);
    sp.layers.push_back(d);
    for (int i = 0; i < n_srcs; ++i) sp.srcs.push_back(srcs[i]);
    sp.n_tiles += (uint32_t)tiles;
    sp.tile_begin.push_back(sp.n_tiles);
    return RANDES_OK;
}

struct Span { uintptr_t lo, hi; int tag; };

// True if any span tagged 0 overlaps any span tagged 1.
bool overlap(std::vector<Span> spans)
{
    // common case first, without sorting: everything tagged 0 lies entirely before or after everything tagged 1
    uintptr_t lo[2] = { ~(uintptr_t)0, ~(uintptr_t)0 }, hi[2] = { 0, 0 };
    for (const Span &s : spans) { lo[s.tag] = std::min(lo[s.tag], s.lo); hi[s.tag] = std::max(hi[s.tag], s.hi); }
    if (hi[0] <= lo[1] || hi[1] <= lo[0]) return false;
    std::sort(spans.begin(), spans.end(), [](const Span &a, const Span &b) { return a.lo < b.lo; });
    uintptr_t hi0 = 0, hi1 = 0;   // furthest end seen so far per tag
    for (const Span &s : spans) {
        if (s.tag == 0) { if (s.lo < hi1) return true; hi0 = std::max(hi0, s.hi); }
        else { if (s.lo < hi0) return true; hi1 = std::max(hi1, s.hi); }
    }
    return false;
}

// True if any two of the spans overlap.
bool any_overlap(std::vector<Span> spans)
{
    auto by_lo = [](const Span &a, const Span &b) { return a.lo < b.lo; };
    if (!std::is_sorted(spans.begin(), spans.end(), by_lo)) std::sort(spans.begin(), spans.end(), by_lo);
    uintptr_t hi = 0;
    for (const Span &s : spans) {
        if (s.lo < hi) return true;
        hi = std::max(hi, s.hi);
    }
    return false;
}

Span span_of(const void *p, size_t elems, int dtype, int tag)
{
    return Span{ (uintptr_t)p, (uintptr_t)p + elems * elem_bytes(dtype), tag };
}

// Every buffer of a call must be memory that HIP knows, reachable from device `dev`, and must lie
// inside its allocation for all the elements the kernels will touch: a kernel handed anything else
// faults the GPU.  Runs when the tables of an argument set are built, not on cached calls; buffers
// that share an allocation (views into one stack) cost one query.
int spans_on_device(const std::vector<Span> &spans, int dev)
{
    uintptr_t known_lo = 0, known_hi = 0;   // allocation of the span checked last
    for (const Span &s : spans) {
        if (s.lo == s.hi || (s.lo >= known_lo && s.hi <= known_hi)) continue;
        hipPointerAttribute_t at;
        hipError_t e = hipPointerGetAttributes(&at, (const void *)s.lo);
        if (e != hipSuccess || at.type == hipMemoryTypeUnregistered) {
            (void)hipGetLastError();
            return fail(RANDES_EINVAL, "a buffer pointer is not memory known to HIP (device memory expected)");
        }
        if (at.type == hipMemoryTypeDevice && at.device != dev)
            return fail(RANDES_EINVAL, "a buffer lies on device " + std::to_string(at.device) +
                                       ", the call was made with device " + std::to_string(dev) + " current");
        void *base = nullptr;
        size_t size = 0;
        e = hipMemGetAddressRange((hipDeviceptr_t *)&base, &size, (hipDeviceptr_t)s.lo);
        if (e != hipSuccess) {      // no range on record for this kind of memory: nothing to compare with
            (void)hipGetLastError();
            known_lo = known_hi = 0;
            continue;
        }
        known_lo = (uintptr_t)base;
        known_hi = known_lo + size;
        if (s.hi > known_hi)
            return fail(RANDES_EINVAL, "a buffer holds fewer elements than its layer's rows x cols: it ends " +
                                       std::to_string(s.hi - known_hi) + " bytes past its allocation");
    }
    return RANDES_OK;
}

}  // namespace

extern "C" {

int randes_layer_perm(uint64_t seed, int32_t group, int32_t group_size, int32_t *perm_out)
{
    if (!perm_out || group_size < 1) return fail(RANDES_EINVAL, "perm_out is NULL or group_size < 1");
    layer_perm(seed, group, group_size, perm_out);
    return RANDES_OK;
}

int randes_source_table(const randes_layer *layers, int32_t n_layers, uint64_t seed, int32_t *src_out)
{
    std::string why;
    int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!src_out) return fail(RANDES_EINVAL, "src_out is NULL");
    std::vector<int32_t> src;
    rc = build_source_table(layers, n_layers, seed, &src, &why);
    if (rc) return fail(rc, why);
    memcpy(src_out, src.data(), sizeof(int32_t) * (size_t)n_layers);
    return RANDES_OK;
}

int randes_sign_mask(uint64_t seed, int32_t layer, int64_t cols, uint8_t *mask_out, void *hip_stream)
{
    if (!mask_out || cols < 1 || layer < 0) return fail(RANDES_EINVAL, "mask_out is NULL, cols < 1 or layer < 0");
    if (cols >= (int64_t)1 << 31) return fail(RANDES_ENOTSUP, "cols >= 2^31");
    hipError_t e = launch_sign_mask((uint32_t)(seed & 0xffffffffu), (uint32_t)(seed >> 32), (uint32_t)layer, cols,
                                    mask_out, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "sign_mask launch");
    return RANDES_OK;
}

}  // extern "C"

namespace {

// compress from deltas (base == NULL) or from fine-tuned weights and the base (deltas formed on the fly)
int merge_impl(const randes_layer *layers, int32_t n_layers,
               const void *const *deltas, const void *const *base, int32_t n_tasks, const uint64_t *seeds,
               randes_dtype delta_dtype, void *const *merged, randes_dtype merged_dtype, void *hip_stream)
{
    std::string why;
    int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!deltas || !seeds || !merged) return fail(RANDES_EINVAL, "deltas, seeds or merged is NULL");
    if (n_tasks < 1) return fail(RANDES_EINVAL, "n_tasks < 1");
    if (n_tasks > RANDES_MAX_TASKS) return fail(RANDES_ENOTSUP, "n_tasks above RANDES_MAX_TASKS");
    if (!dtype_ok(delta_dtype) || !dtype_ok(merged_dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    for (int64_t q = 0; q < (int64_t)n_tasks * n_layers; ++q)
        if (!deltas[q] || !elem_aligned(deltas[q], delta_dtype)) return fail(RANDES_EINVAL, "NULL or misaligned input pointer");
    for (int32_t l = 0; l < n_layers; ++l)
        if (!merged[l] || !elem_aligned(merged[l], merged_dtype) || (base && (!base[l] || !elem_aligned(base[l], delta_dtype))))
            return fail(RANDES_EINVAL, "NULL or misaligned merged or base pointer");

    const Knobs kn = knobs();
    const int32_t head[6] = { base ? PLAN_MERGE_WEIGHTS : PLAN_MERGE, n_layers, n_tasks, (int32_t)delta_dtype,
                              (int32_t)merged_dtype, kn.word(kn.merge_rows) };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(layers, sizeof(randes_layer) * (size_t)n_layers);
    key.add(deltas, sizeof(void *) * (size_t)n_tasks * (size_t)n_layers);
    key.add(seeds, sizeof(uint64_t) * (size_t)n_tasks);
    key.add(merged, sizeof(void *) * (size_t)n_layers);
    if (base) key.add(base, sizeof(void *) * (size_t)n_layers);

    PlanRef cp;
    rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        // the superposition must not overwrite its own inputs
        std::vector<Span> spans;
        for (int32_t l = 0; l < n_layers; ++l) {
            const size_t n = (size_t)layers[l].rows * (size_t)layers[l].cols;
            spans.push_back(span_of(merged[l], n, merged_dtype, 0));
            for (int32_t i = 0; i < n_tasks; ++i) spans.push_back(span_of(deltas[(size_t)i * n_layers + l], n, delta_dtype, 1));
            if (base) spans.push_back(span_of(base[l], n, delta_dtype, 1));
        }
        if (overlap(spans)) return fail(RANDES_EINVAL, "merged overlaps an input");
        if (int bad = spans_on_device(spans, fresh->device)) return bad;

        HostPlan hp;
        std::string why2;
        std::vector<std::vector<int32_t>> src((size_t)n_tasks);
        for (int32_t i = 0; i < n_tasks; ++i) {
            const int rc2 = build_source_table(layers, n_layers, seeds[i], &src[(size_t)i], &why2);
            if (rc2) return fail(rc2, why2);
            hp.keys.push_back((uint32_t)(seeds[i] & 0xffffffffu));
            hp.keys.push_back((uint32_t)(seeds[i] >> 32));
        }
        const int vec = merge_vec(delta_dtype);
        const int n_streams = base ? 2 * n_tasks : n_tasks;
        std::vector<const void *> ptrs((size_t)n_streams);
        for (int32_t l = 0; l < n_layers; ++l) {
            LayerDev d{};
            d.dst = merged[l];
            d.rows = (int32_t)layers[l].rows;
            d.cols = (int32_t)layers[l].cols;
            d.layer_id = (uint32_t)l;
            d.flip = (layers[l].flags & RANDES_FLIP) ? 1u : 0u;
            bool vector_ok = (layers[l].cols % vec) == 0 && aligned16(merged[l]);
            for (int32_t i = 0; i < n_tasks; ++i) {
                ptrs[(size_t)i] = deltas[(size_t)i * n_layers + src[(size_t)i][(size_t)l]];
                vector_ok = vector_ok && aligned16(ptrs[(size_t)i]);
                if (base) {
                    ptrs[(size_t)(n_tasks + i)] = base[src[(size_t)i][(size_t)l]];
                    vector_ok = vector_ok && aligned16(ptrs[(size_t)(n_tasks + i)]);
                }
            }
            const int burst = base ? merge_weights_burst_rows() : merge_burst_rows();
            const StreamBytes eb{ elem_bytes(merged_dtype), 0, 0, elem_bytes(delta_dtype) };
            const int rc2 = place(&hp, d, ptrs.data(), n_streams, vector_ok, vec, clamp_rows(kn.merge_rows, burst), eb);
            if (rc2) return rc2;
        }
        const int rc4 = upload(hp, n_tasks, fresh);
        // 3 to 8 tasks in registers: three waves per SIMD by registers (bf16: all but 8 tasks), two stream
        // faster on long rows (bf16, 16 Llama blocks: 4 tasks +3.3 %, 5 +2.5 %, 6 +1.7 %, 7 +0.8 %; 2 tasks -8 %)
        if (!rc4 && !base && n_tasks >= 3 && n_tasks <= 8)
            fresh->vec.lds_floor = wide_row_lds_floor(hp.vec, elem_bytes(delta_dtype));
        if (!rc4 && !base && (double)n_tasks * stack_bytes(layers, n_layers, delta_dtype) < MERGE_CHUNKED_BELOW_BYTES)
            fresh->vec.xcd_chunk_shift = MERGE_CHUNK_SHIFT;
        return rc4;
    });
    if (rc) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = base ? launch_merge_weights(cp->vec, 1, delta_dtype, merged_dtype, s)
                        : launch_merge(cp->vec, 1, delta_dtype, merged_dtype, s);
    if (e != hipSuccess) return hip_fail(e, "merge launch");
    e = base ? launch_merge_weights(cp->scl, 0, delta_dtype, merged_dtype, s)
             : launch_merge(cp->scl, 0, delta_dtype, merged_dtype, s);
    if (e != hipSuccess) return hip_fail(e, "merge launch (element-wise)");
    return RANDES_OK;
}

}  // namespace

extern "C" {

int randes_merge(const randes_layer *layers, int32_t n_layers,
                 const void *const *deltas, int32_t n_tasks, const uint64_t *seeds,
                 randes_dtype delta_dtype, void *const *merged, randes_dtype merged_dtype, void *hip_stream)
{
    return merge_impl(layers, n_layers, deltas, nullptr, n_tasks, seeds, delta_dtype, merged, merged_dtype, hip_stream);
}

int randes_merge_weights(const randes_layer *layers, int32_t n_layers,
                         const void *const *weights, const void *const *base, int32_t n_tasks, const uint64_t *seeds,
                         randes_dtype weight_dtype, void *const *merged, randes_dtype merged_dtype, void *hip_stream)
{
    if (!base) return fail(RANDES_EINVAL, "base is NULL");
    return merge_impl(layers, n_layers, weights, base, n_tasks, seeds, weight_dtype, merged, merged_dtype, hip_stream);
}

int randes_retrieve(const randes_layer *layers, int32_t n_layers,
                    const void *const *merged, randes_dtype merged_dtype,
                    const void *const *base, randes_dtype base_dtype,
                    uint64_t seed, float lambda,
                    void *const *out, randes_dtype out_dtype, void *hip_stream)
{
    std::string why;
    int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!merged || !base || !out) return fail(RANDES_EINVAL, "merged, base or out is NULL");
    if (!dtype_ok(merged_dtype) || !dtype_ok(base_dtype) || !dtype_ok(out_dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    if (!std::isfinite(lambda)) return fail(RANDES_EINVAL, "lambda is not finite");
    for (int32_t l = 0; l < n_layers; ++l)
        if (!merged[l] || !base[l] || !out[l] || !elem_aligned(merged[l], merged_dtype) ||
            !elem_aligned(base[l], base_dtype) || !elem_aligned(out[l], out_dtype))
            return fail(RANDES_EINVAL, "NULL or misaligned layer pointer");

    const Knobs kn = knobs();
    const int32_t head[6] = { PLAN_RETRIEVE, n_layers, (int32_t)merged_dtype, (int32_t)base_dtype, (int32_t)out_dtype,
                              kn.word(kn.retrieve_rows) };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(layers, sizeof(randes_layer) * (size_t)n_layers);
    key.add(merged, sizeof(void *) * (size_t)n_layers);
    key.add(base, sizeof(void *) * (size_t)n_layers);
    key.add(out, sizeof(void *) * (size_t)n_layers);
    key.add(&seed, sizeof(seed));

    PlanRef cp;
    rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        std::vector<Span> a, b;
        for (int32_t l = 0; l < n_layers; ++l) {
            const size_t n = (size_t)layers[l].rows * (size_t)layers[l].cols;
            a.push_back(span_of(out[l], n, out_dtype, 0));
            a.push_back(span_of(merged[l], n, merged_dtype, 1));
            if (out[l] != base[l] || out_dtype != base_dtype) {
                b.push_back(span_of(out[l], n, out_dtype, 0));
                b.push_back(span_of(base[l], n, base_dtype, 1));
            }
        }
        if (overlap(a)) return fail(RANDES_EINVAL, "out overlaps merged");
        if (overlap(b)) return fail(RANDES_EINVAL, "out partially overlaps base");
        for (int32_t l = 0; l < n_layers; ++l)
            a.push_back(span_of(base[l], (size_t)layers[l].rows * (size_t)layers[l].cols, base_dtype, 1));
        if (int bad = spans_on_device(a, fresh->device)) return bad;

        HostPlan hp;
        std::string why2;
        std::vector<int32_t> src;
        const int rc2 = build_source_table(layers, n_layers, seed, &src, &why2);
        if (rc2) return fail(rc2, why2);
        const int vec = retrieve_vec(merged_dtype, base_dtype);
        const double flipped_bytes = stack_bytes(layers, n_layers, merged_dtype);
        for (int32_t l = 0; l < n_layers; ++l) {
            const int32_t t = src[(size_t)l];
            LayerDev d{};
            d.dst = out[t];
            d.a = merged[l];
            d.b = base[t];
            d.rows = (int32_t)layers[l].rows;
            d.cols = (int32_t)layers[l].cols;
            d.layer_id = (uint32_t)l;
            d.flip = (layers[l].flags & RANDES_FLIP) ? 1u : 0u;
            const bool vector_ok = (layers[l].cols % vec) == 0 && aligned16(d.dst) && aligned16(d.a) && aligned16(d.b);
            const int burst = two_input_burst_rows(merged_dtype, base_dtype, vector_ok ? vec : 1);
            const StreamBytes eb{ elem_bytes(out_dtype), elem_bytes(merged_dtype), elem_bytes(base_dtype), 0 };
            const int rc3 = place(&hp, d, nullptr, 0, vector_ok, vec, two_input_rows_for(kn.retrieve_rows, burst, flipped_bytes, vector_ok), eb);
            if (rc3) return rc3;
        }
        const int rc4 = upload(hp, 1, fresh);
        if (!rc4) fresh->vec.lds_floor = wide_row_lds_floor(hp.vec, elem_bytes(merged_dtype));
        return rc4;
    });
    if (rc) return rc;
    StreamArgs av = cp->vec, as = cp->scl;
    av.key_lo = as.key_lo = (uint32_t)(seed & 0xffffffffu);
    av.key_hi = as.key_hi = (uint32_t)(seed >> 32);
    av.lambda = as.lambda = lambda;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = launch_retrieve(av, 1, merged_dtype, base_dtype, out_dtype, s);
    if (e != hipSuccess) return hip_fail(e, "retrieve launch");
    e = launch_retrieve(as, 0, merged_dtype, base_dtype, out_dtype, s);
    if (e != hipSuccess) return hip_fail(e, "retrieve launch (element-wise)");
    return RANDES_OK;
}

}  // extern "C"

namespace {

// q = 2, 4 or 8 requests in one pass; every layer already known to take the vector path.
int retrieve_many_pass(const randes_layer *layers, int32_t n_layers, const void *const *merged,
                       const void *const *base, int32_t q, const uint64_t *seeds, const float *lambdas,
                       void *const *outs, int dtype, void *hip_stream)
{
    const Knobs kn = knobs();
    const int32_t head[5] = { PLAN_RETRIEVE_MANY, n_layers, dtype, q, kn.word(0) };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(layers, sizeof(randes_layer) * (size_t)n_layers);
    key.add(merged, sizeof(void *) * (size_t)n_layers);
    key.add(base, sizeof(void *) * (size_t)n_layers);
    key.add(outs, sizeof(void *) * (size_t)n_layers * (size_t)q);
    key.add(seeds, sizeof(uint64_t) * (size_t)q);

    PlanRef cp;
    int rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        std::vector<Span> spans;
        for (int32_t l = 0; l < n_layers; ++l) {
            const size_t n = (size_t)layers[l].rows * (size_t)layers[l].cols;
            spans.push_back(span_of(merged[l], n, dtype, 1));
            spans.push_back(span_of(base[l], n, dtype, 1));
            for (int32_t i = 0; i < q; ++i) spans.push_back(span_of(outs[(size_t)i * n_layers + l], n, dtype, 0));
        }
        if (int bad = spans_on_device(spans, fresh->device)) return bad;
        HostPlan hp;
        std::string why;
        std::vector<std::vector<int32_t>> src((size_t)q);
        for (int32_t i = 0; i < q; ++i) {
            const int rc2 = build_source_table(layers, n_layers, seeds[i], &src[(size_t)i], &why);
            if (rc2) return fail(rc2, why);
            hp.keys.push_back((uint32_t)(seeds[i] & 0xffffffffu));
            hp.keys.push_back((uint32_t)(seeds[i] >> 32));
        }
        const int vec = retrieve_vec(dtype, dtype);
        std::vector<const void *> ptrs((size_t)(2 * q));
        for (int32_t l = 0; l < n_layers; ++l) {
            LayerDev d{};
            d.a = merged[l];
            d.rows = (int32_t)layers[l].rows;
            d.cols = (int32_t)layers[l].cols;
            d.layer_id = (uint32_t)l;
            d.flip = (layers[l].flags & RANDES_FLIP) ? 1u : 0u;
            for (int32_t i = 0; i < q; ++i) {
                const int32_t t = src[(size_t)i][(size_t)l];
                ptrs[(size_t)i] = base[t];
                ptrs[(size_t)(q + i)] = outs[(size_t)i * n_layers + t];
            }
            const StreamBytes eb{ 0, elem_bytes(dtype), 0, elem_bytes(dtype) };
            const int rc2 = place(&hp, d, ptrs.data(), 2 * q, true, vec, retrieve_many_rows(q), eb);
            if (rc2) return rc2;
        }
        return upload(hp, q, fresh);
    });
    if (rc) return rc;
    StreamArgs av = cp->vec;
    for (int32_t i = 0; i < q; ++i) av.lambdas[i] = lambdas[i];
    hipError_t e = launch_retrieve_many(av, dtype, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "retrieve (several models) launch");
    return RANDES_OK;
}

}  // namespace

extern "C" {

int randes_retrieve_many(const randes_layer *layers, int32_t n_layers,
                         const void *const *merged, randes_dtype merged_dtype,
                         const void *const *base, randes_dtype base_dtype,
                         int32_t n_requests, const uint64_t *seeds, const float *lambdas,
                         void *const *outs, randes_dtype out_dtype, void *hip_stream)
{
    std::string why;
    int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!merged || !base || !outs || !seeds || !lambdas) return fail(RANDES_EINVAL, "merged, base, outs, seeds or lambdas is NULL");
    if (n_requests < 1) return fail(RANDES_EINVAL, "n_requests < 1");
    if (!dtype_ok(merged_dtype) || !dtype_ok(base_dtype) || !dtype_ok(out_dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    for (int32_t q = 0; q < n_requests; ++q)
        if (!std::isfinite(lambdas[q])) return fail(RANDES_EINVAL, "lambda is not finite");
    const int vec = retrieve_vec(merged_dtype, base_dtype);
    bool vector_ok = merged_dtype == base_dtype && base_dtype == out_dtype;
    std::vector<Span> out_spans, both;
    for (int32_t l = 0; l < n_layers; ++l) {
        if (!merged[l] || !base[l] || !elem_aligned(merged[l], merged_dtype) || !elem_aligned(base[l], base_dtype))
            return fail(RANDES_EINVAL, "NULL or misaligned layer pointer");
        const size_t n = (size_t)layers[l].rows * (size_t)layers[l].cols;
        both.push_back(span_of(merged[l], n, merged_dtype, 1));
        both.push_back(span_of(base[l], n, base_dtype, 1));
        vector_ok = vector_ok && (layers[l].cols % vec) == 0 && aligned16(merged[l]) && aligned16(base[l]);
        for (int32_t q = 0; q < n_requests; ++q) {
            void *o = outs[(size_t)q * n_layers + l];
            if (!o || !elem_aligned(o, out_dtype)) return fail(RANDES_EINVAL, "NULL or misaligned output pointer");
            out_spans.push_back(span_of(o, n, out_dtype, 0));
            both.push_back(out_spans.back());
            vector_ok = vector_ok && aligned16(o);
        }
    }
    if (any_overlap(out_spans)) return fail(RANDES_EINVAL, "output stacks overlap each other");
    if (overlap(both)) return fail(RANDES_EINVAL, "an output overlaps merged or base");
    // geometry limits are the single retrieval's; let it report them
    int32_t q0 = 0;
    while (q0 < n_requests) {
        const int32_t left = n_requests - q0;
        const int32_t q = !vector_ok ? 1 : (left >= 8 ? 8 : (left >= 4 ? 4 : (left >= 2 ? 2 : 1)));
        if (q == 1)
            rc = randes_retrieve(layers, n_layers, merged, merged_dtype, base, base_dtype, seeds[q0], lambdas[q0],
                                 outs + (size_t)q0 * n_layers, out_dtype, hip_stream);
        else
            rc = retrieve_many_pass(layers, n_layers, merged, base, q, seeds + q0, lambdas + q0,
                                    outs + (size_t)q0 * n_layers, (int)merged_dtype, hip_stream);
        if (rc) return rc;
        q0 += q;
    }
    return RANDES_OK;
}

int randes_update(const randes_layer *layers, int32_t n_layers,
                  void *const *merged, randes_dtype merged_dtype,
                  const void *const *delta, randes_dtype delta_dtype,
                  uint64_t seed, int32_t remove, void *hip_stream)
{
    std::string why;
    int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!merged || !delta) return fail(RANDES_EINVAL, "merged or delta is NULL");
    if (!dtype_ok(merged_dtype) || !dtype_ok(delta_dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    for (int32_t l = 0; l < n_layers; ++l)
        if (!merged[l] || !delta[l] || !elem_aligned(merged[l], merged_dtype) || !elem_aligned(delta[l], delta_dtype))
            return fail(RANDES_EINVAL, "NULL or misaligned layer pointer");

    const Knobs kn = knobs();
    const int32_t head[5] = { PLAN_UPDATE, n_layers, (int32_t)merged_dtype, (int32_t)delta_dtype, kn.word(kn.retrieve_rows) };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(layers, sizeof(randes_layer) * (size_t)n_layers);
    key.add(merged, sizeof(void *) * (size_t)n_layers);
    key.add(delta, sizeof(void *) * (size_t)n_layers);
    key.add(&seed, sizeof(seed));

    PlanRef cp;
    rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        std::vector<Span> spans;
        for (int32_t l = 0; l < n_layers; ++l) {
            const size_t n = (size_t)layers[l].rows * (size_t)layers[l].cols;
            spans.push_back(span_of(merged[l], n, merged_dtype, 0));
            spans.push_back(span_of(delta[l], n, delta_dtype, 1));
        }
        if (overlap(spans)) return fail(RANDES_EINVAL, "merged overlaps delta");
        if (int bad = spans_on_device(spans, fresh->device)) return bad;
        HostPlan hp;
        std::string why2;
        std::vector<int32_t> src;
        const int rc2 = build_source_table(layers, n_layers, seed, &src, &why2);
        if (rc2) return fail(rc2, why2);
        const int vec = update_vec(merged_dtype, delta_dtype);
        // In place, the short burst is best at every size (a tile is written back while its DRAM pages are
        // still open): 7B-shaped stack 6.49 ms with 12 rows a wave, 6.38 with 6.
        const double flipped_bytes = 0.0;
        for (int32_t l = 0; l < n_layers; ++l) {
            LayerDev d{};
            d.dst = merged[l];
            d.a = delta[src[(size_t)l]];
            d.rows = (int32_t)layers[l].rows;
            d.cols = (int32_t)layers[l].cols;
            d.layer_id = (uint32_t)l;
            d.flip = (layers[l].flags & RANDES_FLIP) ? 1u : 0u;
            const bool vector_ok = (layers[l].cols % vec) == 0 && aligned16(d.dst) && aligned16(d.a);
            const int burst = two_input_burst_rows(delta_dtype, merged_dtype, vector_ok ? vec : 1);
            const StreamBytes eb{ elem_bytes(merged_dtype), elem_bytes(delta_dtype), 0, 0 };
            const int rc3 = place(&hp, d, nullptr, 0, vector_ok, vec, two_input_rows_for(kn.retrieve_rows, burst, flipped_bytes, vector_ok), eb);
            if (rc3) return rc3;
        }
        const int rc4 = upload(hp, 1, fresh);
        if (!rc4) fresh->vec.lds_floor = wide_row_lds_floor(hp.vec, elem_bytes(merged_dtype));
        return rc4;
    });
    if (rc) return rc;
    StreamArgs av = cp->vec, as = cp->scl;
    av.key_lo = as.key_lo = (uint32_t)(seed & 0xffffffffu);
    av.key_hi = as.key_hi = (uint32_t)(seed >> 32);
    av.negate = as.negate = remove ? 1u : 0u;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = launch_update(av, 1, merged_dtype, delta_dtype, s);
    if (e != hipSuccess) return hip_fail(e, "update launch");
    e = launch_update(as, 0, merged_dtype, delta_dtype, s);
    if (e != hipSuccess) return hip_fail(e, "update launch (element-wise)");
    return RANDES_OK;
}

}  // extern "C"

namespace randes {

int validate_stats_args(const randes_layer *layers, int32_t n_layers,
                        const void *const *delta_a, const void *const *delta_b, int dtype, const double *out3)
{
    std::string why;
    const int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!delta_a || !delta_b || !out3) return fail(RANDES_EINVAL, "delta_a, delta_b or out3 is NULL");
    if (!dtype_ok(dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    for (int32_t l = 0; l < n_layers; ++l)
        if (!delta_a[l] || !delta_b[l] || !elem_aligned(delta_a[l], dtype) || !elem_aligned(delta_b[l], dtype))
            return fail(RANDES_EINVAL, "NULL or misaligned layer pointer");
    if (((uintptr_t)out3 & 7u) != 0) return fail(RANDES_EINVAL, "out3 is not 8-byte aligned");
    return RANDES_OK;
}

int build_stats_plan(const randes_layer *layers, int32_t n_layers,
                     const void *const *delta_a, uint64_t seed_a,
                     const void *const *delta_b, uint64_t seed_b,
                     int dtype, HostPlan *hp)
{
    std::string why;
    int rc;
    const Knobs kn = knobs();
    std::vector<int32_t> sa, sb;
    if ((rc = build_source_table(layers, n_layers, seed_a, &sa, &why))) return fail(rc, why);
    if ((rc = build_source_table(layers, n_layers, seed_b, &sb, &why))) return fail(rc, why);
    const int vec = stats_vec(dtype);
    for (int32_t l = 0; l < n_layers; ++l) {
        LayerDev d{};
        d.a = delta_a[sa[(size_t)l]];
        d.b = delta_b[sb[(size_t)l]];
        d.rows = (int32_t)layers[l].rows;
        d.cols = (int32_t)layers[l].cols;
        d.layer_id = (uint32_t)l;
        d.flip = (layers[l].flags & RANDES_FLIP) ? 1u : 0u;
        const bool vector_ok = (layers[l].cols % vec) == 0 && aligned16(d.a) && aligned16(d.b);
        const int burst = two_input_burst_rows(dtype, dtype, vector_ok ? vec : 1);
        const StreamBytes eb{ 0, elem_bytes(dtype), elem_bytes(dtype), 0 };
        if ((rc = place(hp, d, nullptr, 0, vector_ok, vec, clamp_rows(kn.retrieve_rows, burst), eb))) return rc;
    }
    hp->extra_bytes = ((size_t)hp->vec.n_tiles + hp->scl.n_tiles) * 3 * sizeof(double);
    return RANDES_OK;
}

}  // namespace randes

extern "C" {

int randes_delta_stats(const randes_layer *layers, int32_t n_layers,
                       const void *const *delta_a, uint64_t seed_a,
                       const void *const *delta_b, uint64_t seed_b,
                       randes_dtype dtype, double *out3, void *hip_stream)
{
    int rc = validate_stats_args(layers, n_layers, delta_a, delta_b, dtype, out3);
    if (rc) return rc;
    const Knobs kn = knobs();
    // The per-workgroup partial sums live with the tables, and calls on one stream run in order:
    // one set of tables per stream keeps equal calls on different streams apart.
    const int32_t head[4] = { PLAN_STATS, n_layers, (int32_t)dtype, kn.word(kn.retrieve_rows) };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(layers, sizeof(randes_layer) * (size_t)n_layers);
    key.add(delta_a, sizeof(void *) * (size_t)n_layers);
    key.add(delta_b, sizeof(void *) * (size_t)n_layers);
    key.add(&seed_a, sizeof(seed_a));
    key.add(&seed_b, sizeof(seed_b));
    key.add(&hip_stream, sizeof(hip_stream));

    PlanRef cp;
    rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        std::vector<Span> spans;
        for (int32_t l = 0; l < n_layers; ++l) {
            const size_t n = (size_t)layers[l].rows * (size_t)layers[l].cols;
            spans.push_back(span_of(delta_a[l], n, dtype, 1));
            spans.push_back(span_of(delta_b[l], n, dtype, 1));
        }
        spans.push_back(Span{ (uintptr_t)out3, (uintptr_t)out3 + 3 * sizeof(double), 0 });
        if (int bad = spans_on_device(spans, fresh->device)) return bad;
        HostPlan hp;
        const int rc2 = build_stats_plan(layers, n_layers, delta_a, seed_a, delta_b, seed_b, dtype, &hp);
        if (rc2) return rc2;
        return upload(hp, 1, fresh);
    });
    if (rc) return rc;
    StreamArgs av = cp->vec, as = cp->scl;
    av.key_lo = as.key_lo = (uint32_t)(seed_a & 0xffffffffu);
    av.key_hi = as.key_hi = (uint32_t)(seed_a >> 32);
    av.key2_lo = as.key2_lo = (uint32_t)(seed_b & 0xffffffffu);
    av.key2_hi = as.key2_hi = (uint32_t)(seed_b >> 32);
    av.partials = as.partials = (double *)cp->extra;
    av.partial_base = 0;
    as.partial_base = av.n_tiles;
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = launch_stats(av, 1, dtype, s);
    if (e != hipSuccess) return hip_fail(e, "stats launch");
    e = launch_stats(as, 0, dtype, s);
    if (e != hipSuccess) return hip_fail(e, "stats launch (element-wise)");
    e = launch_stats_finalize((const double *)cp->extra, av.n_tiles + as.n_tiles, out3, s);
    if (e != hipSuccess) return hip_fail(e, "stats finalize launch");
    return RANDES_OK;
}

}  // extern "C"

namespace {

// Tables of a LoRA launch: choose the band shape, cut the matrices into workgroup tiles, upload.
int build_lora_tables(std::vector<LoraItem> &items, const std::vector<LoraSeg> &segs, int32_t rank, int ab_dtype,
                      CachedPlan *fresh)
{
    uint64_t tiles = 0;
    uint32_t max_seg = 1;
    bool fast = (rank % 8) == 0;
    for (const LoraItem &it : items) {
        max_seg = std::max(max_seg, it.n_seg);
        fast = fast && (it.cols % 8) == 0 && aligned16(it.out);
        // the wide path addresses with 32-bit byte offsets inside a matrix
        fast = fast && (int64_t)it.rows * it.cols < ((int64_t)1 << 30) && (int64_t)it.rows * rank < ((int64_t)1 << 30) &&
               (int64_t)it.cols * rank < ((int64_t)1 << 30);
    }
    for (const LoraSeg &sg : segs) fast = fast && aligned16(sg.A) && aligned16(sg.B);
    const LoraShape shape = lora_choose_shape(items.data(), items.size(), (int32_t)max_seg, rank, ab_dtype == RANDES_F32, fast);
    const int64_t wg_rows = (int64_t)32 * shape.rt * shape.rb;
    for (LoraItem &it : items) {
        it.tiles_x = (uint32_t)(((int64_t)it.cols + shape.tile_cols - 1) / shape.tile_cols);
        it.tile_begin = (uint32_t)tiles;
        tiles += (uint64_t)it.tiles_x * (uint64_t)(((int64_t)it.rows + wg_rows - 1) / wg_rows);
        if (tiles >= ((uint64_t)1 << 31)) return fail(RANDES_ENOTSUP, "too many tiles for one launch");
    }
    const size_t items_bytes = (sizeof(LoraItem) * items.size() + 255) & ~(size_t)255;
    const size_t segs_bytes = (sizeof(LoraSeg) * segs.size() + 255) & ~(size_t)255;
    std::vector<char> host(items_bytes + segs_bytes + (size_t)tiles * sizeof(uint32_t), 0);
    memcpy(host.data(), items.data(), sizeof(LoraItem) * items.size());
    memcpy(host.data() + items_bytes, segs.data(), sizeof(LoraSeg) * segs.size());
    uint32_t *wg_item = (uint32_t *)(host.data() + items_bytes + segs_bytes);
    for (size_t q = 0; q < items.size(); ++q) {
        const uint64_t end = q + 1 < items.size() ? items[q + 1].tile_begin : tiles;
        for (uint64_t t = items[q].tile_begin; t < end; ++t) wg_item[t] = (uint32_t)q;
    }
    hipError_t e = hipMalloc(&fresh->blob, host.size());
    if (e != hipSuccess) { fresh->blob = nullptr; return hip_fail(e, "hipMalloc(lora tables)"); }
    fresh->blob_bytes = host.size();
    e = hipMemcpy(fresh->blob, host.data(), host.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) { (void)hipFree(fresh->blob); fresh->blob = nullptr; return hip_fail(e, "hipMemcpy(lora tables)"); }
    fresh->items_bytes = items_bytes;
    fresh->segs_bytes = segs_bytes;
    fresh->lora_tiles = (uint32_t)tiles;
    fresh->lora_shape = shape;
    fresh->lora_fast = fast;
    return RANDES_OK;
}

int launch_cached_lora(const CachedPlan &cp, int32_t rank, float scale, int ab_dtype, int out_dtype, void *hip_stream)
{
    hipError_t e = launch_lora((const LoraItem *)cp.blob, (const LoraSeg *)((const char *)cp.blob + cp.items_bytes),
                               (const uint32_t *)((const char *)cp.blob + cp.items_bytes + cp.segs_bytes), cp.lora_tiles,
                               cp.lora_shape, cp.lora_fast, rank, scale, ab_dtype, out_dtype, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "lora launch");
    return RANDES_OK;
}

}  // namespace

extern "C" {

int randes_lora_materialize_batched(int32_t n, const void *const *Bs, const void *const *As,
                                    const int64_t *rows, const int64_t *cols, int32_t rank,
                                    float scale, randes_dtype ab_dtype,
                                    void *const *outs, randes_dtype out_dtype, void *hip_stream)
{
    if (n < 1 || !Bs || !As || !rows || !cols || !outs) return fail(RANDES_EINVAL, "NULL array or n < 1");
    if (rank < 1) return fail(RANDES_EINVAL, "rank < 1");
    if (!dtype_ok(ab_dtype) || !dtype_ok(out_dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    if (!std::isfinite(scale)) return fail(RANDES_EINVAL, "scale is not finite");
    for (int32_t q = 0; q < n; ++q) {
        if (!Bs[q] || !As[q] || !outs[q]) return fail(RANDES_EINVAL, "NULL matrix pointer");
        if (!elem_aligned(Bs[q], ab_dtype) || !elem_aligned(As[q], ab_dtype) || !elem_aligned(outs[q], out_dtype))
            return fail(RANDES_EINVAL, "misaligned matrix pointer");
        if (rows[q] < 1 || cols[q] < 1) return fail(RANDES_EINVAL, "rows < 1 or cols < 1");
        if (rows[q] >= (int64_t)1 << 31 || cols[q] >= (int64_t)1 << 31) return fail(RANDES_ENOTSUP, "rows or cols >= 2^31");
    }
    // workgroups read factors while others write outputs: nothing written may be a factor or another output
    // (swept when the argument set is first seen; equal arguments give an equal verdict)
    std::vector<Span> both;
    auto no_overlap = [&]() -> int {
        std::vector<Span> out_spans;
        for (int32_t q = 0; q < n; ++q) {
            out_spans.push_back(span_of(outs[q], (size_t)rows[q] * (size_t)cols[q], out_dtype, 0));
            both.push_back(out_spans.back());
            both.push_back(span_of(Bs[q], (size_t)rows[q] * (size_t)rank, ab_dtype, 1));
            both.push_back(span_of(As[q], (size_t)rank * (size_t)cols[q], ab_dtype, 1));
        }
        if (any_overlap(out_spans)) return fail(RANDES_EINVAL, "output matrices overlap each other");
        if (overlap(both)) return fail(RANDES_EINVAL, "an output matrix overlaps a factor");
        return RANDES_OK;
    };
    const int32_t head[5] = { PLAN_LORA, n, rank, (int32_t)ab_dtype, (int32_t)out_dtype };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(Bs, sizeof(void *) * (size_t)n);
    key.add(As, sizeof(void *) * (size_t)n);
    key.add(rows, sizeof(int64_t) * (size_t)n);
    key.add(cols, sizeof(int64_t) * (size_t)n);
    key.add(outs, sizeof(void *) * (size_t)n);
    PlanRef cp;
    int rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        if (int bad = spans_on_device(both, fresh->device)) return bad;
        std::vector<LoraItem> items((size_t)n);
        std::vector<LoraSeg> segs((size_t)n);
        for (int32_t q = 0; q < n; ++q) {
            LoraItem &it = items[(size_t)q];
            memset(&it, 0, sizeof(it));
            it.out = outs[q];
            it.rows = (int32_t)rows[q]; it.cols = (int32_t)cols[q];
            it.seg_begin = (uint32_t)q; it.n_seg = 1;
            LoraSeg &sg = segs[(size_t)q];
            memset(&sg, 0, sizeof(sg));
            sg.B = Bs[q]; sg.A = As[q];
        }
        return build_lora_tables(items, segs, rank, ab_dtype, fresh);
    }, no_overlap);
    if (rc) return rc;
    return launch_cached_lora(*cp, rank, scale, ab_dtype, out_dtype, hip_stream);
}

int randes_lora_merge(const randes_layer *layers, int32_t n_layers,
                      const void *const *Bs, const void *const *As, int32_t rank,
                      int32_t n_tasks, const uint64_t *seeds, float scale, randes_dtype ab_dtype,
                      void *const *merged, randes_dtype merged_dtype, void *hip_stream)
{
    std::string why;
    int rc = validate_layers(layers, n_layers, &why);
    if (rc) return fail(rc, why);
    if (!Bs || !As || !seeds || !merged) return fail(RANDES_EINVAL, "Bs, As, seeds or merged is NULL");
    if (n_tasks < 1 || rank < 1) return fail(RANDES_EINVAL, "n_tasks < 1 or rank < 1");
    if (n_tasks > RANDES_MAX_TASKS) return fail(RANDES_ENOTSUP, "n_tasks above RANDES_MAX_TASKS");
    if (!dtype_ok(ab_dtype) || !dtype_ok(merged_dtype)) return fail(RANDES_EINVAL, "unknown dtype");
    if (!std::isfinite(scale)) return fail(RANDES_EINVAL, "scale is not finite");
    for (int64_t q = 0; q < (int64_t)n_tasks * n_layers; ++q)
        if (!Bs[q] || !As[q] || !elem_aligned(Bs[q], ab_dtype) || !elem_aligned(As[q], ab_dtype))
            return fail(RANDES_EINVAL, "NULL or misaligned factor pointer");
    for (int32_t l = 0; l < n_layers; ++l)
        if (!merged[l] || !elem_aligned(merged[l], merged_dtype)) return fail(RANDES_EINVAL, "NULL or misaligned merged pointer");
    for (int32_t l = 0; l < n_layers; ++l)
        if (layers[l].rows >= (int64_t)1 << 31) return fail(RANDES_ENOTSUP, "rows >= 2^31");
    std::vector<Span> both;
    auto no_overlap = [&]() -> int {   // swept when the argument set is first seen
        std::vector<Span> out_spans;
        for (int32_t l = 0; l < n_layers; ++l) {
            const size_t rows = (size_t)layers[l].rows, cols = (size_t)layers[l].cols;
            out_spans.push_back(span_of(merged[l], rows * cols, merged_dtype, 0));
            both.push_back(out_spans.back());
            for (int32_t i = 0; i < n_tasks; ++i) {
                both.push_back(span_of(Bs[(size_t)i * n_layers + l], rows * (size_t)rank, ab_dtype, 1));
                both.push_back(span_of(As[(size_t)i * n_layers + l], (size_t)rank * cols, ab_dtype, 1));
            }
        }
        if (any_overlap(out_spans)) return fail(RANDES_EINVAL, "merged matrices overlap each other");
        if (overlap(both)) return fail(RANDES_EINVAL, "a merged matrix overlaps a factor");
        return RANDES_OK;
    };
    const int32_t head[6] = { PLAN_LORA_MERGE, n_layers, n_tasks, rank, (int32_t)ab_dtype, (int32_t)merged_dtype };
    CallKey key;
    key.add(head, sizeof(head));
    key.add(layers, sizeof(randes_layer) * (size_t)n_layers);
    key.add(Bs, sizeof(void *) * (size_t)n_tasks * (size_t)n_layers);
    key.add(As, sizeof(void *) * (size_t)n_tasks * (size_t)n_layers);
    key.add(seeds, sizeof(uint64_t) * (size_t)n_tasks);
    key.add(merged, sizeof(void *) * (size_t)n_layers);
    PlanRef cp;
    rc = find_or_build(key, hip_stream, &cp, [&](CachedPlan *fresh) -> int {
        if (int bad = spans_on_device(both, fresh->device)) return bad;
        std::string why2;
        std::vector<std::vector<int32_t>> src((size_t)n_tasks);
        for (int32_t i = 0; i < n_tasks; ++i) {
            const int rc2 = build_source_table(layers, n_layers, seeds[i], &src[(size_t)i], &why2);
            if (rc2) return fail(rc2, why2);
        }
        std::vector<LoraItem> items((size_t)n_layers);
        std::vector<LoraSeg> segs;
        segs.reserve((size_t)n_layers * (size_t)n_tasks);
        for (int32_t l = 0; l < n_layers; ++l) {
            LoraItem &it = items[(size_t)l];
            memset(&it, 0, sizeof(it));
            it.out = merged[l];
            it.rows = (int32_t)layers[l].rows; it.cols = (int32_t)layers[l].cols;
            it.seg_begin = (uint32_t)segs.size(); it.n_seg = (uint32_t)n_tasks;
            for (int32_t i = 0; i < n_tasks; ++i) {
                LoraSeg sg;
                memset(&sg, 0, sizeof(sg));
                const int32_t t = src[(size_t)i][(size_t)l];
                sg.B = Bs[(size_t)i * n_layers + t];
                sg.A = As[(size_t)i * n_layers + t];
                sg.key_lo = (uint32_t)(seeds[i] & 0xffffffffu);
                sg.key_hi = (uint32_t)(seeds[i] >> 32);
                sg.layer_id = (uint32_t)l;
                sg.flip = (layers[l].flags & RANDES_FLIP) ? 1u : 0u;
                segs.push_back(sg);
            }
        }
        return build_lora_tables(items, segs, rank, ab_dtype, fresh);
    }, no_overlap);
    if (rc) return rc;
    return launch_cached_lora(*cp, rank, scale, ab_dtype, merged_dtype, hip_stream);
}

int randes_lora_materialize(const void *B, const void *A, int64_t rows, int64_t cols, int32_t rank,
                            float scale, randes_dtype ab_dtype,
                            void *delta_out, randes_dtype out_dtype, void *hip_stream)
{
    return randes_lora_materialize_batched(1, &B, &A, &rows, &cols, rank, scale, ab_dtype, &delta_out, out_dtype, hip_stream);
}

const char *randes_strerror(int code)
{
    switch (code) {
    case RANDES_OK: return "ok";
    case RANDES_EINVAL: return g_detail.empty() ? "invalid argument" : g_detail.c_str();
    case RANDES_ENOTSUP: return g_detail.empty() ? "not supported" : g_detail.c_str();
    case RANDES_EHIP: return g_detail.empty() ? "HIP runtime failure" : g_detail.c_str();
    default: return "unknown error code";
    }
}

int randes_shutdown(void)
{
    std::lock_guard<std::mutex> lock(g_mu);
    int rc = RANDES_OK;
    for (const PlanRef &cp : g_lru) {
        if (cp->blob) {
            hipError_t e = hipFree(cp->blob);
            if (e != hipSuccess) rc = hip_fail(e, "hipFree(plan tables)");
            cp->blob = nullptr;
        }
    }
    for (const PlanRef &cp : g_retired) {
        if (!cp->blob) continue;
        hipError_t e = hipFree(cp->blob);
        if (e != hipSuccess) rc = hip_fail(e, "hipFree(retired plan tables)");
        cp->blob = nullptr;
    }
    g_retired.clear();
    g_retired_bytes = 0;
    g_index.clear();
    g_lru.clear();
    g_pinned = 0;
    return rc;
}

// ------------------------------------------------------------------ measurement aids (randes_bench.h)
int randes_set_tile_rows(int32_t merge_rows, int32_t retrieve_rows)
{
    if (merge_rows < 0 || retrieve_rows < 0 || merge_rows > (1 << 20) || retrieve_rows > (1 << 20))
        return fail(RANDES_EINVAL, "tile rows out of range");
    knobs().merge_rows = merge_rows;
    knobs().retrieve_rows = retrieve_rows;
    return RANDES_OK;
}

int randes_probe_stream(const void *const *inputs, int32_t n_inputs, void *output, int64_t bytes, int32_t write,
                        void *hip_stream)
{
    if (!inputs || !output || n_inputs < 1 || n_inputs > 8) return fail(RANDES_EINVAL, "inputs/output NULL or n_inputs outside 1..8");
    if (bytes < (int64_t)PROBE_CHUNK_BYTES || bytes % (int64_t)PROBE_CHUNK_BYTES) return fail(RANDES_EINVAL, "bytes must be a positive multiple of 16384");
    if (bytes / (int64_t)PROBE_CHUNK_BYTES >= (int64_t)1 << 31) return fail(RANDES_ENOTSUP, "stream too long for one launch");
    for (int32_t k = 0; k < n_inputs; ++k)
        if (!inputs[k] || !aligned16(inputs[k])) return fail(RANDES_EINVAL, "NULL or unaligned input stream");
    if (!aligned16(output)) return fail(RANDES_EINVAL, "unaligned output");
    hipError_t e = launch_probe(inputs, n_inputs, output, (uint64_t)bytes, write, (hipStream_t)hip_stream);
    if (e != hipSuccess) return hip_fail(e, "probe launch");
    return RANDES_OK;
}

int randes_set_tile_cols(int32_t max_waves_along_columns)
{
    int shift;
    switch (max_waves_along_columns) {
    case 0: case 4: shift = 2; break;
    case 2: shift = 1; break;
    case 1: shift = 0; break;
    default: return fail(RANDES_EINVAL, "max_waves_along_columns must be 0, 1, 2 or 4");
    }
    knobs().max_wx_shift = shift;
    return RANDES_OK;
}

int randes_set_fold(int32_t enable)
{
    knobs().fold = enable ? 1 : 0;
    return RANDES_OK;
}

}  // extern "C"
