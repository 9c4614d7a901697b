// Placement of the stacks of a serving set-up in device memory: the host logic that finds the
// memory's address groups from copy rates and packs stacks into them, and the timing of the copies.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <map>
#include <string>
#include <vector>

#include "../../include/randes_place.h"
#include "api_internal.hpp"
#include "launch.hpp"

namespace randes {
namespace {

// Centres of a two-cluster split of the values (medians, so that a few outliers do not become a
// cluster of their own); false if one cluster is empty.
bool two_medians(std::vector<double> vals, double *lo_out, double *hi_out)
{
    std::sort(vals.begin(), vals.end());
    const size_t n = vals.size();
    if (n == 0) return false;
    double lo = vals[n / 10], hi = vals[n - 1 - n / 10];
    for (int it = 0; it < 8; ++it) {
        const double mid = 0.5 * (lo + hi);
        const size_t a = (size_t)(std::lower_bound(vals.begin(), vals.end(), mid) - vals.begin());   // values below mid
        if (a == 0 || a == n) return false;
        lo = vals[a / 2];
        hi = vals[a + (n - a) / 2];
    }
    *lo_out = lo;
    *hi_out = hi;
    return true;
}

// Middle element of the longest run of consecutive numbers in an ascending list (the first such run).
int32_t middle_of_longest_run(const std::vector<int32_t> &chunks)
{
    size_t best_begin = 0, best_len = 0, cur_begin = 0;
    for (size_t i = 0; i < chunks.size(); ++i) {
        if (i > 0 && chunks[i] != chunks[i - 1] + 1) cur_begin = i;
        const size_t len = i - cur_begin + 1;
        if (len > best_len) { best_len = len; best_begin = cur_begin; }
    }
    return chunks[best_begin + best_len / 2];
}

struct Run { int32_t group, first, end; };

std::vector<Run> runs_of(const int32_t *labels, int32_t n)
{
    std::vector<Run> out;
    int32_t start = 0;
    for (int32_t c = 1; c <= n; ++c)
        if (c == n || labels[c] != labels[start]) { out.push_back(Run{ labels[start], start, c }); start = c; }
    return out;
}

uint64_t align_up(uint64_t x) { return (x + 255u) / 256u * 256u; }

struct Range { int32_t group; uint64_t lo, hi; };

struct DeviceRates {
    char *arena;
    uint64_t chunk_bytes;
    hipStream_t stream;
    hipEvent_t a, b;
    hipError_t err;
};

double device_rate(int32_t r, int32_t w, void *ctx)
{
    DeviceRates *d = (DeviceRates *)ctx;
    if (d->err != hipSuccess) return 0.0;
    const void *in = d->arena + (uint64_t)r * d->chunk_bytes;
    void *out = d->arena + (uint64_t)w * d->chunk_bytes;
    float best = -1.0f;
    for (int i = 0; i < 5; ++i) {   // the first launch warms up
        hipError_t e = hipEventRecord(d->a, d->stream);
        if (e == hipSuccess) e = launch_probe(&in, 1, out, d->chunk_bytes, 1, d->stream);
        if (e == hipSuccess) e = hipEventRecord(d->b, d->stream);
        if (e == hipSuccess) e = hipEventSynchronize(d->b);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, d->a, d->b);
        if (e != hipSuccess) { d->err = e; return 0.0; }
        if (i > 0 && (best < 0.0f || ms < best)) best = ms;
    }
    return best > 0.0f ? 2.0 * (double)d->chunk_bytes / (double)best : 0.0;
}

}  // namespace
}  // namespace randes

using namespace randes;

extern "C" {

int randes_place_classify(int32_t n_chunks, randes_copy_rate_fn rate, void *ctx,
                          double min_separation, int32_t max_groups, int32_t *labels_out)
{
    if (n_chunks < 1 || !rate || !labels_out) return fail(RANDES_EINVAL, "n_chunks < 1, or rate or labels_out is NULL");
    if (min_separation <= 0.0) min_separation = 0.02;
    if (max_groups <= 0) max_groups = 4;
    std::vector<int32_t> rest((size_t)n_chunks);
    for (int32_t c = 0; c < n_chunks; ++c) { labels_out[c] = -1; rest[(size_t)c] = c; }
    int32_t g = 0;
    while (rest.size() > 1 && g < max_groups - 1) {
        const int32_t ref = middle_of_longest_run(rest);
        std::map<int32_t, double> rates;
        std::vector<double> values;
        for (const int32_t c : rest)
            if (c != ref) { const double v = rate(ref, c, ctx); rates[c] = v; values.push_back(v); }
        double lo, hi;
        if (!two_medians(values, &lo, &hi) || (hi - lo) / hi < min_separation) break;
        const double mid = 0.5 * (lo + hi);
        std::map<int32_t, int> other;   // 1: copies fast from the reference, so lies in another group
        for (const auto &kv : rates) other[kv.first] = kv.second >= mid ? 1 : 0;
        other[ref] = 0;
        std::map<int32_t, int> voted;
        size_t ones = 0;
        for (const int32_t c : rest) {
            int sum = 0, cnt = 0;
            for (int32_t x = c - 2; x <= c + 2; ++x) {
                const auto f = other.find(x);
                if (f != other.end()) { sum += f->second; ++cnt; }
            }
            const int v = 2 * sum > cnt ? 1 : 0;
            voted[c] = v;
            ones += (size_t)v;
        }
        if (std::min(ones, rest.size() - ones) < 3) break;   // not a group, a handful of misreads
        std::vector<int32_t> next;
        for (const int32_t c : rest) {
            if (voted[c] == 0) labels_out[c] = g;
            else next.push_back(c);
        }
        rest.swap(next);
        ++g;
    }
    for (const int32_t c : rest) labels_out[c] = g;
    return RANDES_OK;
}

int randes_place_classify_device(void *arena, uint64_t chunk_bytes, int32_t n_chunks, void *hip_stream,
                                 int32_t *labels_out)
{
    if (!arena || !labels_out || n_chunks < 1) return fail(RANDES_EINVAL, "arena or labels_out is NULL, or n_chunks < 1");
    if (chunk_bytes < PROBE_CHUNK_BYTES || chunk_bytes % PROBE_CHUNK_BYTES) return fail(RANDES_EINVAL, "chunk_bytes must be a positive multiple of 16384");
    if (chunk_bytes / PROBE_CHUNK_BYTES >= (uint64_t)1 << 31) return fail(RANDES_ENOTSUP, "chunk too long for one launch");
    if (!aligned16(arena)) return fail(RANDES_EINVAL, "arena is not 16-byte aligned");
    DeviceRates d;
    d.arena = (char *)arena;
    d.chunk_bytes = chunk_bytes;
    d.stream = (hipStream_t)hip_stream;
    d.err = hipSuccess;
    hipError_t e = hipEventCreate(&d.a);
    if (e != hipSuccess) return hip_fail(e, "hipEventCreate");
    e = hipEventCreate(&d.b);
    if (e != hipSuccess) { (void)hipEventDestroy(d.a); return hip_fail(e, "hipEventCreate"); }
    const int rc = randes_place_classify(n_chunks, device_rate, &d, 0.0, 0, labels_out);
    (void)hipEventDestroy(d.a);
    (void)hipEventDestroy(d.b);
    if (d.err != hipSuccess) return hip_fail(d.err, "timed copy");
    return rc;
}

int randes_place_serving_layout(const int32_t *labels, int32_t n_chunks, uint64_t chunk_bytes,
                                uint64_t stack_bytes, int32_t n_models, int32_t n_more_outputs,
                                uint64_t *offsets_out, int32_t *groups_out)
{
    if (!labels || !offsets_out || !groups_out || n_chunks < 1 || chunk_bytes < 1 || stack_bytes < 1 || n_models < 0 ||
        n_more_outputs < 0)
        return fail(RANDES_EINVAL, "NULL array, or a count or size below its minimum");
    const std::vector<Run> rs = runs_of(labels, n_chunks);
    std::vector<int32_t> groups;
    for (int32_t c = 0; c < n_chunks; ++c) groups.push_back(labels[c]);
    std::sort(groups.begin(), groups.end());
    groups.erase(std::unique(groups.begin(), groups.end()), groups.end());
    if (groups.size() < 3) return fail(RANDES_ENOTSUP, "fewer than three address groups");
    const uint64_t half = align_up(stack_bytes / 2);

    for (size_t i = 0; i + 1 < rs.size(); ++i) {
        const Run &r1 = rs[i], &r2 = rs[i + 1];
        const uint64_t edge = (uint64_t)r1.end * chunk_bytes;
        // half a stack and a chunk of margin on both sides of the boundary
        if ((uint64_t)(r1.end - r1.first) * chunk_bytes < half + chunk_bytes ||
            (uint64_t)(r2.end - r2.first) * chunk_bytes < half + chunk_bytes)
            continue;
        const uint64_t out_off = edge - half, out_end = out_off + align_up(stack_bytes);
        for (const int32_t read_group : groups) {
            if (read_group == r1.group || read_group == r2.group) continue;
            // (group, lo, hi) byte ranges usable for whole stacks
            std::vector<Range> fr;
            for (size_t q = 0; q < rs.size(); ++q) {
                uint64_t lo = (uint64_t)rs[q].first * chunk_bytes + (rs[q].first > 0 ? chunk_bytes : 0);
                uint64_t hi = (uint64_t)rs[q].end * chunk_bytes;
                const uint64_t margin = rs[q].end < n_chunks ? chunk_bytes : 0;
                hi = hi > margin ? hi - margin : 0;
                if (q == i) hi = std::min((uint64_t)rs[q].end * chunk_bytes, out_off);            // left of the straddled boundary
                if (q == i + 1) lo = std::max((uint64_t)rs[q].first * chunk_bytes, out_end);     // right of it
                if (hi > lo) fr.push_back(Range{ rs[q].group, align_up(lo), hi });
            }
            auto take = [&](bool want_read_group, uint64_t *off) {
                for (Range &r : fr)
                    if ((r.group == read_group) == want_read_group && r.lo + stack_bytes <= r.hi) {
                        *off = r.lo;
                        r.lo = align_up(r.lo + stack_bytes);
                        return true;
                    }
                return false;
            };
            std::vector<uint64_t> offs((size_t)(3 + n_models + n_more_outputs));
            bool ok = take(true, &offs[0]) && take(true, &offs[1]);
            offs[2] = out_off;
            for (int32_t m = 0; ok && m < n_models + n_more_outputs; ++m) ok = take(false, &offs[(size_t)(3 + m)]);
            if (!ok) continue;
            std::copy(offs.begin(), offs.end(), offsets_out);
            groups_out[0] = read_group;
            groups_out[1] = r1.group;
            groups_out[2] = r2.group;
            return RANDES_OK;
        }
    }
    return fail(RANDES_ENOTSUP, "the address groups found do not hold this layout");
}

}  // extern "C"
