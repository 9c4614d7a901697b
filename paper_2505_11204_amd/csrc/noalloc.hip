// randes_delta_stats_noalloc: the Sec. 3 diagnostics for callers that cannot allocate device memory
// (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).
//
// The ordinary entry point keeps two things in device memory of its own: the descriptor tables of
// the call and one triple of partial sums per workgroup.  Here both live in `scratch`, a fixed
// array that is part of the library's code object, and the tables reach it inside kernel arguments
// (poke_kernel), so the call consists of kernel launches only: no hipMalloc, no hipFree, no
// hipMemcpy.  The streaming and the final reduction are the ordinary entry point's kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <vector>

#include "api_internal.hpp"
#include "device_util.hpp"
#include "launch.hpp"

namespace randes {

constexpr size_t SCRATCH_BYTES = (size_t)8 << 20;        // per GPU, held until the process ends
constexpr size_t SCRATCH_TABLE_BYTES = (size_t)1 << 20;  // descriptor tables of one call
constexpr size_t SCRATCH_PARTIAL_BYTES = SCRATCH_BYTES - SCRATCH_TABLE_BYTES;   // 24 bytes per workgroup

// Layout: [0, SCRATCH_TABLE_BYTES) tables of the last call, then the partial sums of the last call.
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static unsigned char *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each GPU, once looked up

// The address of this GPU's copy of the array (the symbol's name is not a device address in host code).
static int scratch_address(unsigned char **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(RANDES_ENOTSUP, "device ordinal above 63");
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = (unsigned char *)p;
    }
    *out = g_scratch_ptr[dev];
    return RANDES_OK;
}

// Kernel arguments carry up to POKE_WORDS dwords of a table image to their place in device memory.
constexpr uint32_t POKE_WORDS = 960;   // 3840 bytes of payload; with the header below the 4 KB of kernel arguments
struct PokeArgs {
    uint32_t *dst;
    uint32_t n_words;
    uint32_t pad;
    uint32_t word[POKE_WORDS];
};

__global__ void __launch_bounds__(WG) poke_kernel(const PokeArgs a)
{
    for (uint32_t q = threadIdx.x; q < a.n_words; q += WG) a.dst[q] = a.word[q];
}

}  // namespace randes

using namespace randes;

extern "C" int randes_delta_stats_noalloc(const randes_layer *layers, int32_t n_layers,
                                          const void *const *delta_a, uint64_t seed_a,
                                          const void *const *delta_b, uint64_t seed_b,
                                          randes_dtype dtype, double *out3, void *hip_stream)
{
    int rc = validate_stats_args(layers, n_layers, delta_a, delta_b, dtype, out3);
    if (rc) return rc;
    HostPlan hp;
    if ((rc = build_stats_plan(layers, n_layers, delta_a, seed_a, delta_b, seed_b, dtype, &hp))) return rc;
    std::vector<char> image;
    TableLayout lay;
    pack_tables(hp, &image, &lay);
    if (image.size() > SCRATCH_TABLE_BYTES)
        return fail(RANDES_ENOTSUP, "randes_delta_stats_noalloc: the call's descriptor tables exceed the 1 MiB the fixed "
                                    "scratch array reserves for them (too many layers); use randes_delta_stats");
    if (hp.extra_bytes > SCRATCH_PARTIAL_BYTES)
        return fail(RANDES_ENOTSUP, "randes_delta_stats_noalloc: the call needs more than 305834 workgroups (about 10^10 "
                                    "bf16 or 5 * 10^9 f32 elements), whose partial sums exceed the 7 MiB the fixed "
                                    "scratch array reserves for them; use randes_delta_stats");
    unsigned char *base = nullptr;
    if ((rc = scratch_address(&base))) return rc;

    hipStream_t s = (hipStream_t)hip_stream;
    // tables: 256-byte aligned pieces of the image, through kernel arguments
    PokeArgs pa;
    const size_t n_words = (image.size() + 3) / 4;
    image.resize(n_words * 4, 0);
    for (size_t w0 = 0; w0 < n_words; w0 += POKE_WORDS) {
        const size_t n = std::min<size_t>(POKE_WORDS, n_words - w0);
        pa.dst = (uint32_t *)base + w0;
        pa.n_words = (uint32_t)n;
        pa.pad = 0;
        memcpy(pa.word, image.data() + w0 * 4, n * 4);
        hipLaunchKernelGGL(poke_kernel, dim3(1), dim3(WG), 0, s, pa);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(e, "table launch");
    }
    // Nothing in the array has to start at zero: every workgroup of the two launches below writes its
    // own triple before the final reduction reads exactly those triples.
    StreamArgs av, as;
    bind_tables(base, lay, hp, 1, &av, &as);
    double *partials = (double *)(base + SCRATCH_TABLE_BYTES);
    av.key_lo = as.key_lo = (uint32_t)(seed_a & 0xffffffffu);
    av.key_hi = as.key_hi = (uint32_t)(seed_a >> 32);
    av.key2_lo = as.key2_lo = (uint32_t)(seed_b & 0xffffffffu);
    av.key2_hi = as.key2_hi = (uint32_t)(seed_b >> 32);
    av.partials = as.partials = partials;
    av.partial_base = 0;
    as.partial_base = av.n_tiles;
    hipError_t e = launch_stats(av, 1, dtype, s);
    if (e != hipSuccess) return hip_fail(e, "stats launch");
    e = launch_stats(as, 0, dtype, s);
    if (e != hipSuccess) return hip_fail(e, "stats launch (element-wise)");
    e = launch_stats_finalize(partials, av.n_tiles + as.n_tiles, out3, s);
    if (e != hipSuccess) return hip_fail(e, "stats finalize launch");
    return RANDES_OK;
}
