// gfx950 streaming kernels of the RanDeS hot path: merge (compress, from deltas or straight from
// weights), fused retrieve, in-place hot-swap update, the Sec. 3 diagnostics, the sign-mask dump,
// and a plain bandwidth probe.  Wavefronts are 64 lanes; a workgroup is 4 waves.
//
// One workgroup owns a tile = (slot layer, a few rows, a block of columns).  A lane owns VEC
// adjacent columns (one 16-byte access per row and stream).  Each wave does ONE burst: it issues
// every load of its rows back to back, the workgroup produces the tile's sign bits (Sec. 4.4: D
// is diagonal over the columns, so bits depend on the column only) into LDS while those loads are
// in flight, then the wave does its arithmetic and issues all its stores last.  The weight stream
// goes HBM -> registers -> HBM and never touches LDS; the sign flip is an XOR on the loaded words.
// The shuffle (Sec. 4.3) costs nothing here: it is already folded into the pointer tables.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "device_util.hpp"
#include "launch.hpp"
#include "philox.hpp"

namespace randes {

template <int DT, int VEC> struct NumWords {
    static constexpr int value = (DT == DT_F32) ? VEC : (VEC == 1 ? 1 : VEC / 2);
};

// Load VEC elements of dtype DT from byte address p as raw dwords (bf16 stays packed).
template <int DT, int VEC>
__device__ __forceinline__ void load_raw(gcptr p, uint32_t (&raw)[NumWords<DT, VEC>::value])
{
    constexpr int NW = NumWords<DT, VEC>::value;
    if constexpr (NW == 1) {
        if constexpr (DT == DT_F32) raw[0] = __builtin_nontemporal_load((const RANDES_GLOBAL uint32_t *)p);
        else raw[0] = (uint32_t)__builtin_nontemporal_load((const RANDES_GLOBAL uint16_t *)p);
    } else if constexpr (NW == 2) {
        const u32x2 q = __builtin_nontemporal_load((const RANDES_GLOBAL u32x2 *)p);
        raw[0] = q.x; raw[1] = q.y;
    } else {
#pragma unroll
        for (int h = 0; h < NW / 4; ++h) {
            const u32x4 q = __builtin_nontemporal_load((const RANDES_GLOBAL u32x4 *)p + h);
            raw[4 * h + 0] = q.x; raw[4 * h + 1] = q.y; raw[4 * h + 2] = q.z; raw[4 * h + 3] = q.w;
        }
    }
}

// Raw dwords -> VEC binary32 values (bf16 widens exactly).
template <int DT, int VEC>
__device__ __forceinline__ void widen(const uint32_t (&raw)[NumWords<DT, VEC>::value], float (&v)[VEC])
{
    if constexpr (DT == DT_F32) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) v[j] = u2f(raw[j]);
    } else if constexpr (VEC == 1) {
        v[0] = u2f(raw[0] << 16);
    } else {
#pragma unroll
        for (int j = 0; j < VEC / 2; ++j) {
            v[2 * j] = u2f(raw[j] << 16);
            v[2 * j + 1] = u2f(raw[j] & 0xffff0000u);
        }
    }
}

// One register per task: this lane's sign bits arranged so that a shift and an AND give the XOR
// mask of any raw dword.  f32: bit j is element j.  bf16 pairs: the even elements' bits sit at
// 12..15 and the odd elements' at 28..31, so dword j uses (W << (3 - j)) & 0x80008000.
template <int DT, int VEC>
__device__ __forceinline__ uint32_t sign_word(uint32_t bits)
{
    if constexpr (DT == DT_F32 || VEC == 1) {
        return bits;
    } else {
        uint32_t e = bits & 0x55u, o = (bits >> 1) & 0x55u;
        e = (e | (e >> 1)) & 0x33u; e = (e | (e >> 2)) & 0x0fu;
        o = (o | (o >> 1)) & 0x33u; o = (o | (o >> 2)) & 0x0fu;
        return (e << 12) | (o << 28);
    }
}

// XOR mask of raw dword j out of the sign word: flips the sign of every element of the dword whose bit is set.
template <int DT, int VEC>
__device__ __forceinline__ uint32_t flip_mask(uint32_t W, int j)
{
    if constexpr (DT == DT_F32) return (W << (31 - j)) & 0x80000000u;
    else if constexpr (VEC == 1) return (W & 1u) << 15;
    else return (W << (3 - j)) & 0x80008000u;
}

// acc[j] += (+/-) x[j] with the masks rebuilt from the sign word (keeps registers for loads).
template <int DT, int VEC>
__device__ __forceinline__ void accumulate_w(const uint32_t (&raw)[NumWords<DT, VEC>::value], uint32_t W, float (&acc)[VEC])
{
    constexpr int NW = NumWords<DT, VEC>::value;
    uint32_t t[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) t[j] = raw[j] ^ flip_mask<DT, VEC>(W, j);
    float v[VEC];
    widen<DT, VEC>(t, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = acc[j] + v[j];
}

// The same with the XOR masks of the raw dwords handed in ready-made.
template <int DT, int VEC>
__device__ __forceinline__ void accumulate_m(const uint32_t (&raw)[NumWords<DT, VEC>::value],
                                             const uint32_t (&mask)[NumWords<DT, VEC>::value], float (&acc)[VEC])
{
    constexpr int NW = NumWords<DT, VEC>::value;
    uint32_t t[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) t[j] = raw[j] ^ mask[j];
    float v[VEC];
    widen<DT, VEC>(t, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = acc[j] + v[j];
}

// acc[j] += (+/-) (theta[j] - base[j]): the delta Delta_i = Theta_i - Theta_0 (Sec. 3) formed in
// binary32 on the fly, one rounding, then flipped and added like a stored delta.
template <int DT, int VEC>
__device__ __forceinline__ void accumulate_sub(const uint32_t (&rt)[NumWords<DT, VEC>::value],
                                               const uint32_t (&rb)[NumWords<DT, VEC>::value], uint32_t bits,
                                               float (&acc)[VEC])
{
    float th[VEC], ba[VEC];
    widen<DT, VEC>(rt, th);
    widen<DT, VEC>(rb, ba);
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        const float d = th[j] - ba[j];
        acc[j] = acc[j] + u2f(f2u(d) ^ ((bits << (31 - j)) & 0x80000000u));
    }
}

// Workgroup barrier that waits for LDS traffic only, so global loads issued before it stay in flight.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Pack VEC binary32 results into the words that go to memory (bf16: RNE, two per word).
template <int DT, int VEC> struct OutWords {
    static constexpr int value = (DT == DT_F32) ? VEC : (VEC == 1 ? 1 : VEC / 2);
};

template <int DT, int VEC>
__device__ __forceinline__ void pack_out(const float (&v)[VEC], uint32_t (&w)[OutWords<DT, VEC>::value])
{
    if constexpr (DT == DT_F32) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) w[j] = f2u(v[j]);
    } else if constexpr (VEC == 1) {
        w[0] = bf16_rne(v[0]);
    } else {
#pragma unroll
        for (int j = 0; j < VEC / 2; ++j) w[j] = pack_bf16x2(v[2 * j], v[2 * j + 1]);
    }
}

template <int DT, int VEC>
__device__ __forceinline__ void store_words(gptr p, const uint32_t (&w)[OutWords<DT, VEC>::value])
{
    constexpr int NW = OutWords<DT, VEC>::value;
    if constexpr (NW == 1) {
        if constexpr (DT == DT_F32) __builtin_nontemporal_store(w[0], (RANDES_GLOBAL uint32_t *)p);
        else __builtin_nontemporal_store((uint16_t)w[0], (RANDES_GLOBAL uint16_t *)p);
    } else if constexpr (NW == 2) {
        u32x2 q;
        q.x = w[0]; q.y = w[1];
        __builtin_nontemporal_store(q, (RANDES_GLOBAL u32x2 *)p);
    } else {
#pragma unroll
        for (int h = 0; h < NW / 4; ++h) {
            u32x4 q;
            q.x = w[4 * h]; q.y = w[4 * h + 1]; q.z = w[4 * h + 2]; q.w = w[4 * h + 3];
            __builtin_nontemporal_store(q, (RANDES_GLOBAL u32x4 *)p + h);
        }
    }
}

// Keeps every store of a burst behind every load of the burst: a wave that first
// issues all its loads and then all its stores sustains markedly more HBM
// bandwidth on this chip than one that alternates them.
__device__ __forceinline__ void load_store_fence() { asm volatile("" ::: "memory"); }

// Where this workgroup works.
struct Tile {
    LayerDev L;
    int layer_slot;       // index into the sub-plan's layer array
    uint32_t col;         // first column of this lane
    uint32_t col_in_tile;
    uint32_t tile_col0;   // first column of the workgroup's tile
    uint32_t cw;          // columns of the workgroup's tile
    uint32_t row0, row_end;
    uint32_t wy, WY;      // this wave's place among the WY waves of the workgroup that are stacked along the rows
    bool active;          // lane has columns inside the layer
    bool valid;           // false: this workgroup is padding of the XCD-contiguous grid and has no tile
    uint32_t id;          // position of the tile in the launch's tile sequence
};

constexpr uint32_t N_XCD = 8;   // workgroup i of a launch is dispatched to XCD i mod 8

// Launch size for n_tiles tiles: a multiple of the XCD count, or of a round of chunks (see locate()).
static inline uint32_t xcd_grid(uint32_t n_tiles, uint32_t chunk_shift = 0)
{
    const uint32_t q = N_XCD << chunk_shift;
    return (n_tiles + q - 1u) / q * q;
}

template <int VEC>
__device__ __forceinline__ Tile locate(const StreamArgs &A)
{
    // Workgroups are handed to the 8 XCDs round-robin.  Give XCD x the x-th contiguous eighth of the
    // tile sequence, so that each XCD (own L2, own address-translation cache) sweeps one region of
    // every stream front to back instead of touching all of them: measured +5..8 % bandwidth.
    // With chunks (A.xcd_chunk_shift = s > 0) the XCDs take runs of 1 << s tiles in turn instead: all of
    // them then work in the same stretch of the stack and finish together, whatever the tiles cost.
    const uint32_t xi = blockIdx.x / N_XCD, xcd = blockIdx.x % N_XCD, cs = A.xcd_chunk_shift;
    const uint32_t bid = cs ? ((((xi >> cs) * N_XCD + xcd) << cs) + (xi & ((1u << cs) - 1u)))
                            : xcd * (gridDim.x / N_XCD) + xi;
    Tile t;
    t.valid = bid < A.n_tiles;
    t.id = bid;
    if (!t.valid) return t;
    // coarse[i] = layer that holds tile i * 1024: narrows the search to a step or two
    int lo = (int)A.coarse[bid >> 10], hi = (int)A.coarse[(bid >> 10) + 1] + 1;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (A.tile_begin[mid] <= bid) lo = mid; else hi = mid;
    }
    t.layer_slot = lo;
    t.L = A.layers[lo];
    const uint32_t idx = bid - A.tile_begin[lo];
    const uint32_t cb = idx % t.L.n_cb, rc = idx / t.L.n_cb;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wx = wave & (t.L.wx - 1u);
    t.WY = (uint32_t)WAVES >> t.L.wx_shift;
    t.wy = wave >> t.L.wx_shift;
    t.cw = t.L.wx * 64u * VEC;
    t.col_in_tile = (wx * 64u + lane) * VEC;
    t.tile_col0 = cb * t.cw;
    t.col = t.tile_col0 + t.col_in_tile;
    t.active = t.col < (uint32_t)t.L.cols;
    t.row0 = rc * t.L.tile_rows;
    const uint32_t re = t.row0 + t.L.tile_rows;
    t.row_end = re < (uint32_t)t.L.rows ? re : (uint32_t)t.L.rows;
    return t;
}

// The workgroup produces the sign bits of its tile's columns once, cooperatively,
// into LDS: sbits[(task * nblk + blk) * 4 + word] for the generator blocks that
// cover [tile_col0, tile_col0 + cw).  A tile may start in the middle of a
// 128-column block (element-wise kernels), so bits are addressed relative to the
// block that contains the tile's first column.  Returns nblk.  Caller barriers.
__device__ __forceinline__ uint32_t stage_sign_bits(uint32_t *sbits, const Tile &t, const uint32_t *keys,
                                                    uint32_t n_keys, uint32_t key_lo, uint32_t key_hi)
{
    const uint32_t lead = t.tile_col0 & 127u;
    const uint32_t nblk = (lead + t.cw + 127u) / 128u;
    if (t.L.flip) {
        for (uint32_t q = threadIdx.x; q < n_keys * nblk; q += WG) {
            const uint32_t i = q / nblk, blk = q % nblk;
            const uint32_t klo = keys ? keys[2 * i] : key_lo, khi = keys ? keys[2 * i + 1] : key_hi;
            uint32_t gen_blk = (t.tile_col0 >> 7) + blk;
            if (t.L.sign_blocks) gen_blk %= t.L.sign_blocks;   // folded rows: the pattern of one row repeats
            const u32x4_t o = sign_block(klo, khi, t.L.layer_id, gen_blk);
            uint32_t *w = sbits + (size_t)q * 4u;
            w[0] = o.w[0]; w[1] = o.w[1]; w[2] = o.w[2]; w[3] = o.w[3];
        }
    }
    return nblk;
}

// This lane's VEC sign bits of task i, out of the staged words.
template <int VEC>
__device__ __forceinline__ uint32_t lane_bits_from_lds(const uint32_t *sbits, const Tile &t, uint32_t nblk, uint32_t i)
{
    if (!t.L.flip) return 0u;
    const uint32_t rel = (t.tile_col0 & 127u) + t.col_in_tile;
    constexpr uint32_t vm = (VEC == 32) ? 0xffffffffu : ((1u << VEC) - 1u);
    return (sbits[(size_t)i * nblk * 4u + (rel >> 5)] >> (rel & 31u)) & vm;
}

// ---------------------------------------------------------------------------
// compress: merged[l] = sum_i D_i^l-flipped delta_i[src_i(l)], binary32, task order.
// A wave owns R rows of its column slice per burst.  It first issues the loads of
// all R rows of all tasks, and while they are in flight the workgroup produces
// its sign bits; then it accumulates and only then stores the R result rows.
// KT > 0: exactly KT tasks, every load of the burst in flight at once.
// KT = 0: any number of tasks, loaded eight at a time for two rows.
// ---------------------------------------------------------------------------
// SUB: the inputs are weights, not deltas: task i contributes Theta_i[src] - Theta_0[src]; the
// source table then holds, per slot layer, the T fine-tuned pointers followed by the T base pointers.
template <int DTI, int DTO, int VEC, int KT, int R, bool SUB>
__global__ void __launch_bounds__(WG) merge_kernel(const StreamArgs A)
{
    constexpr int NW = NumWords<DTI, VEC>::value, NWO = OutWords<DTO, VEC>::value;
    constexpr uint32_t EBI = (DTI == DT_F32) ? 4 : 2, EBO = (DTO == DT_F32) ? 4 : 2;
    constexpr int NS = SUB ? 2 : 1;                          // input streams per task
    extern __shared__ uint32_t sbits[];
    __shared__ gcptr sptr[KT > 0 ? 1 : NS * RANDES_MAX_TASKS];   // KT = 0: tile base pointer of every stream
    const Tile t = locate<VEC>(A);
    if (!t.valid) return;   // whole workgroup, before any barrier
    const uint32_t K = KT > 0 ? (uint32_t)KT : (uint32_t)A.n_tasks;
    const uint32_t rb_in = (uint32_t)t.L.cols * EBI, rb_out = (uint32_t)t.L.cols * EBO;
    const size_t tile_in = (size_t)t.row0 * rb_in, tile_out = (size_t)t.row0 * rb_out;
    // A wave owns R consecutive rows of the tile (rows of one stream lie next to each other in memory,
    // and so do the pieces a wave reads of it: measured 1.3 % faster than rows interleaved over the waves).
    uint32_t off_in = t.wy * R * rb_in + t.col * EBI;
    uint32_t off_out = t.wy * R * rb_out + t.col * EBO;
    const uint32_t step_in = rb_in, step_out = rb_out;
    const gptr dst = (gptr)t.L.dst + tile_out;

    if constexpr (KT > 0) {
        gcptr src[NS * KT];
#pragma unroll
        for (int i = 0; i < NS * KT; ++i) src[i] = (gcptr)A.srcs[(size_t)t.layer_slot * (NS * KT) + i] + tile_in;
        uint32_t raw[R][NS * KT][NW];
        const uint32_t r = t.row0 + t.wy * R;
        // first burst's loads go out before the sign bits exist
        if (t.active) {
            // task by task, the rows of one task together: measured 1.7 % faster than row by row
#pragma unroll
            for (int i = 0; i < NS * KT; ++i)
#pragma unroll
                for (int j = 0; j < R; ++j)
                    if (r + j < t.row_end) load_raw<DTI, VEC>(src[i] + (off_in + j * step_in), raw[j][i]);
        }
        const uint32_t nblk = stage_sign_bits(sbits, t, A.keys, K, 0u, 0u);
        lds_barrier();
        if (!t.active) return;
        uint32_t W[KT];
#pragma unroll
        for (int i = 0; i < KT; ++i) {
            const uint32_t bits = lane_bits_from_lds<VEC>(sbits, t, nblk, i);
            W[i] = SUB ? bits : sign_word<DTI, VEC>(bits);
        }
        // bf16 pairs: every task's XOR masks made once and kept in registers for all R rows (the asm
        // keeps the compiler from rebuilding them row by row, which it otherwise prefers); a raw dword
        // then costs one XOR, and the widening of its two halves folds into it.
        constexpr bool MASKS = !SUB && DTI == DT_BF16 && VEC > 1;
        uint32_t M[MASKS ? KT : 1][NW];
        if constexpr (MASKS) {
#pragma unroll
            for (int i = 0; i < KT; ++i)
#pragma unroll
                for (int q = 0; q < NW; ++q) {
                    M[i][q] = flip_mask<DTI, VEC>(W[i], q);
                    asm volatile("" : "+v"(M[i][q]));
                }
        }
        // The plan gives a wave at most R rows of a tile, so this one burst is all its work.
        uint32_t res[R][NWO];
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (r + j < t.row_end) {
                float acc[VEC];
#pragma unroll
                for (int q = 0; q < VEC; ++q) acc[q] = 0.0f;
#pragma unroll
                for (int i = 0; i < KT; ++i) {
                    if constexpr (SUB) accumulate_sub<DTI, VEC>(raw[j][i], raw[j][KT + i], W[i], acc);
                    else if constexpr (MASKS) accumulate_m<DTI, VEC>(raw[j][i], M[i], acc);
                    else accumulate_w<DTI, VEC>(raw[j][i], W[i], acc);
                }
                pack_out<DTO, VEC>(acc, res[j]);
            }
        load_store_fence();
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (r + j < t.row_end) store_words<DTO, VEC>(dst + (off_out + j * step_out), res[j]);
    } else {
        const uint32_t nblk = stage_sign_bits(sbits, t, A.keys, K, 0u, 0u);
        for (uint32_t i = threadIdx.x; i < NS * K; i += WG)
            sptr[i] = (gcptr)A.srcs[(size_t)t.layer_slot * (NS * K) + i] + tile_in;
        __syncthreads();
        if (!t.active) return;
        constexpr int KC = SUB ? 4 : 8;   // tasks loaded per step
        // The plan gives a wave at most R rows of a tile.
        const uint32_t r = t.row0 + t.wy * R;
        if (r < t.row_end) {
            uint32_t res[R][NWO];
#pragma unroll
            for (int j0 = 0; j0 < R; j0 += 2) {
                const bool ok0 = r + j0 < t.row_end;
                const bool ok1 = (j0 + 1 < R) && (r + j0 + 1 < t.row_end);
                if (ok0) {
                    float acc[2][VEC];
#pragma unroll
                    for (int u = 0; u < 2; ++u)
#pragma unroll
                        for (int q = 0; q < VEC; ++q) acc[u][q] = 0.0f;
                    for (uint32_t i0 = 0; i0 < K; i0 += KC) {
                        uint32_t raw[2][NS * KC][NW];
#pragma unroll
                        for (int q = 0; q < KC; ++q) {
                            if (i0 + q < K) {
#pragma unroll
                                for (int st = 0; st < NS; ++st) {
                                    const gcptr p = sptr[st * K + i0 + q] + (off_in + j0 * step_in);
                                    load_raw<DTI, VEC>(p, raw[0][st * KC + q]);
                                    if (ok1) load_raw<DTI, VEC>(p + step_in, raw[1][st * KC + q]);
                                }
                            }
                        }
#pragma unroll
                        for (int q = 0; q < KC; ++q) {
                            if (i0 + q < K) {
                                const uint32_t bits = lane_bits_from_lds<VEC>(sbits, t, nblk, i0 + q);
                                if constexpr (SUB) {
                                    accumulate_sub<DTI, VEC>(raw[0][q], raw[0][KC + q], bits, acc[0]);
                                    if (ok1) accumulate_sub<DTI, VEC>(raw[1][q], raw[1][KC + q], bits, acc[1]);
                                } else {
                                    const uint32_t W = sign_word<DTI, VEC>(bits);
                                    uint32_t Mq[NW];   // one set of masks for both rows (see M above)
#pragma unroll
                                    for (int w = 0; w < NW; ++w) {
                                        Mq[w] = flip_mask<DTI, VEC>(W, w);
                                        if constexpr (DTI == DT_BF16 && VEC > 1) asm volatile("" : "+v"(Mq[w]));
                                    }
                                    accumulate_m<DTI, VEC>(raw[0][q], Mq, acc[0]);
                                    if (ok1) accumulate_m<DTI, VEC>(raw[1][q], Mq, acc[1]);
                                }
                            }
                        }
                    }
                    pack_out<DTO, VEC>(acc[0], res[j0]);
                    if (j0 + 1 < R) pack_out<DTO, VEC>(acc[1], res[j0 + 1 < R ? j0 + 1 : j0]);
                }
            }
            load_store_fence();
#pragma unroll
            for (int j = 0; j < R; ++j)
                if (r + j < t.row_end) store_words<DTO, VEC>(dst + (off_out + j * step_out), res[j]);
        }
    }
}

// ---------------------------------------------------------------------------
// Two-input bursts shared by retrieve and hot-swap update:
//   retrieve: out[t] = fma(lambda, D-flipped merged[l], base[t]),  t = src(l)
//   update:   merged[l] <- merged[l] + (+/-) D-flipped delta[src(l)]
// X is the stream the sign flip acts on, Y the other input.  Same shape as the
// merge: loads of R rows, sign bits while they fly, arithmetic, then R stores.
// ---------------------------------------------------------------------------
template <int DTX, int DTY, int DTO, int VEC, bool FMA>
__device__ __forceinline__ void two_input_bursts(const StreamArgs &A, const Tile &t, gcptr px, gcptr py,
                                                 gptr po, uint32_t *sbits)
{
    constexpr uint32_t EBX = (DTX == DT_F32) ? 4 : 2, EBY = (DTY == DT_F32) ? 4 : 2, EBO = (DTO == DT_F32) ? 4 : 2;
    constexpr int NWX = NumWords<DTX, VEC>::value, NWY = NumWords<DTY, VEC>::value, NWO = OutWords<DTO, VEC>::value;
    constexpr int R = two_input_rows(NWX, NWY);
    const uint32_t cols = (uint32_t)t.L.cols;
    px += (size_t)t.row0 * cols * EBX;
    py += (size_t)t.row0 * cols * EBY;
    po += (size_t)t.row0 * cols * EBO;
    // Rows of a tile are dealt to the waves in turn (wave wy owns rows wy, wy + WY, ...): with two
    // read streams this measured 1 % faster than consecutive rows per wave, the merge's arrangement.
    const uint32_t e = t.wy * cols + t.col;         // element offset inside the tile (times 4 stays below 2^32)
    const uint32_t estep = t.WY * cols;
    const uint32_t r = t.row0 + t.wy;
    uint32_t rx[R][NWX], ry[R][NWY];
    if (t.active) {
        // one stream after the other: measured 0.5 % faster than row by row
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + t.WY * u < t.row_end) load_raw<DTX, VEC>(px + (e + u * estep) * EBX, rx[u]);
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + t.WY * u < t.row_end) load_raw<DTY, VEC>(py + (e + u * estep) * EBY, ry[u]);
    }
    const uint32_t nblk = stage_sign_bits(sbits, t, nullptr, 1u, A.key_lo, A.key_hi);
    lds_barrier();
    if (!t.active) return;
    uint32_t bits = lane_bits_from_lds<VEC>(sbits, t, nblk, 0u);
    if (A.negate) bits = ~bits;
    // The flip acts on X's raw dwords (bf16: one XOR per pair of elements), with the masks made once per lane.
    uint32_t xm[NWX];
    {
        const uint32_t W = sign_word<DTX, VEC>(bits);
#pragma unroll
        for (int j = 0; j < NWX; ++j) xm[j] = flip_mask<DTX, VEC>(W, j);
    }
    const float lambda = A.lambda;
    // The plan gives a wave at most R rows of a tile, so this one burst is all its work.
    uint32_t res[R][NWO];
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (r + t.WY * u < t.row_end) {
            float x[VEC], y[VEC], o[VEC];
            uint32_t fx[NWX];
#pragma unroll
            for (int j = 0; j < NWX; ++j) fx[j] = rx[u][j] ^ xm[j];
            widen<DTX, VEC>(fx, x);
            widen<DTY, VEC>(ry[u], y);
#pragma unroll
            for (int j = 0; j < VEC; ++j) o[j] = FMA ? __builtin_fmaf(lambda, x[j], y[j]) : (y[j] + x[j]);
            pack_out<DTO, VEC>(o, res[u]);
        }
    load_store_fence();
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (r + t.WY * u < t.row_end) store_words<DTO, VEC>(po + (e + u * estep) * EBO, res[u]);
}

template <int DTM, int DTB, int DTO, int VEC>
__global__ void __launch_bounds__(WG) retrieve_kernel(const StreamArgs A)
{
    extern __shared__ uint32_t sbits[];
    const Tile t = locate<VEC>(A);
    if (!t.valid) return;
    two_input_bursts<DTM, DTB, DTO, VEC, true>(A, t, (gcptr)t.L.a, (gcptr)t.L.b, (gptr)t.L.dst, sbits);
}

// ---------------------------------------------------------------------------
// Several retrievals in one pass: for Q models at once,
//   out_q[t_q] = fma(lambda_q, D_q-flipped merged[l], base[t_q]),  t_q = src_q(l),
// each bit-identical to the single retrieval.  The merged tile is read once for all Q models
// (the base tiles are not shared: under model q's permutation slot l maps to its own layer t_q).
// The source table holds, per slot layer, the Q base pointers followed by the Q output pointers.
// Mirror image of the merge: 1 + Q read streams, Q write streams; all loads of the burst, the
// sign bits while they fly, the arithmetic in place over the base registers, then all stores.
// ---------------------------------------------------------------------------
template <int DT, int VEC, int QT>
__global__ void __launch_bounds__(WG) retrieve_many_kernel(const StreamArgs A)
{
    constexpr int NW = NumWords<DT, VEC>::value;
    static_assert(NW == OutWords<DT, VEC>::value, "results replace the base registers word for word");
    constexpr uint32_t EB = (DT == DT_F32) ? 4 : 2;
    constexpr int R = retrieve_many_rows(QT);
    extern __shared__ uint32_t sbits[];
    const Tile t = locate<VEC>(A);
    if (!t.valid) return;   // whole workgroup, before any barrier
    const uint32_t cols = (uint32_t)t.L.cols;
    const size_t tile_off = (size_t)t.row0 * cols * EB;
    const gcptr pm = (gcptr)t.L.a + tile_off;
    gcptr pb[QT];
    gptr po[QT];
#pragma unroll
    for (int q = 0; q < QT; ++q) {
        pb[q] = (gcptr)A.srcs[(size_t)t.layer_slot * (2 * QT) + q] + tile_off;
        po[q] = (gptr)A.srcs[(size_t)t.layer_slot * (2 * QT) + QT + q] + tile_off;
    }
    const uint32_t off = (t.wy * R * cols + t.col) * EB, step = cols * EB;   // bytes inside the tile, below 2^32; consecutive rows
    const uint32_t r = t.row0 + t.wy * R;
    uint32_t rm[R][NW], ry[R][QT][NW];
    if (t.active) {
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + u < t.row_end) load_raw<DT, VEC>(pm + (off + u * step), rm[u]);
#pragma unroll
        for (int q = 0; q < QT; ++q)
#pragma unroll
            for (int u = 0; u < R; ++u)
                if (r + u < t.row_end) load_raw<DT, VEC>(pb[q] + (off + u * step), ry[u][q]);
    }
    const uint32_t nblk = stage_sign_bits(sbits, t, A.keys, (uint32_t)QT, 0u, 0u);
    lds_barrier();
    if (!t.active) return;
    uint32_t bits[QT];
#pragma unroll
    for (int q = 0; q < QT; ++q) bits[q] = lane_bits_from_lds<VEC>(sbits, t, nblk, (uint32_t)q);
    // The plan gives a wave at most R rows of a tile, so this one burst is all its work.
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (r + u < t.row_end) {
            float x[VEC];
            widen<DT, VEC>(rm[u], x);
#pragma unroll
            for (int q = 0; q < QT; ++q) {
                float y[VEC], o[VEC];
                widen<DT, VEC>(ry[u][q], y);
                const float lambda = A.lambdas[q];
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    const float xs = u2f(f2u(x[j]) ^ ((bits[q] << (31 - j)) & 0x80000000u));
                    o[j] = __builtin_fmaf(lambda, xs, y[j]);
                }
                pack_out<DT, VEC>(o, ry[u][q]);
            }
        }
    load_store_fence();
#pragma unroll
    for (int q = 0; q < QT; ++q)
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + u < t.row_end) store_words<DT, VEC>(po[q] + (off + u * step), ry[u][q]);
}

// hot swap: the flipped stream is the delta; the other input and the output are merged[l].
template <int DTM, int DTD, int VEC>
__global__ void __launch_bounds__(WG) update_kernel(const StreamArgs A)
{
    extern __shared__ uint32_t sbits[];
    const Tile t = locate<VEC>(A);
    if (!t.valid) return;
    two_input_bursts<DTD, DTM, DTM, VEC, false>(A, t, (gcptr)t.L.a, (gcptr)t.L.dst, (gptr)t.L.dst, sbits);
}

// ---------------------------------------------------------------------------
// Diagnostics of Sec. 3 ("Interference in Model Merging"): inner product and squared norms of two
// transformed deltas a' = D_a-flipped a[src_a(l)], b' = D_b-flipped b[src_b(l)] over a whole stack,
// in binary64.  Same burst shape as retrieve (two read streams, no write stream); each workgroup
// leaves one triple in `partials`, summed afterwards in a fixed order, so the result does not
// depend on scheduling.
// ---------------------------------------------------------------------------
template <int DT, int VEC>
__global__ void __launch_bounds__(WG) stats_kernel(const StreamArgs A)
{
    constexpr uint32_t EB = (DT == DT_F32) ? 4 : 2;
    constexpr int NW = NumWords<DT, VEC>::value;
    constexpr int R = two_input_rows(NW, NW);
    extern __shared__ uint32_t sbits[];
    __shared__ double swave[WAVES][3];
    const Tile t = locate<VEC>(A);
    if (!t.valid) return;
    const uint32_t cols = (uint32_t)t.L.cols;
    const gcptr pa = (gcptr)t.L.a + (size_t)t.row0 * cols * EB;
    const gcptr pb = (gcptr)t.L.b + (size_t)t.row0 * cols * EB;
    const uint32_t e = t.wy * cols + t.col, estep = t.WY * cols;   // rows dealt to the waves in turn, as in retrieve
    const uint32_t r = t.row0 + t.wy;
    uint32_t ra[R][NW], rb[R][NW];
    if (t.active) {
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + t.WY * u < t.row_end) load_raw<DT, VEC>(pa + (e + u * estep) * EB, ra[u]);
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + t.WY * u < t.row_end) load_raw<DT, VEC>(pb + (e + u * estep) * EB, rb[u]);
    }
    const uint32_t nblk = stage_sign_bits(sbits, t, nullptr, 1u, A.key_lo, A.key_hi);
    stage_sign_bits(sbits + nblk * 4u, t, nullptr, 1u, A.key2_lo, A.key2_hi);
    lds_barrier();
    double s_ab = 0.0, s_aa = 0.0, s_bb = 0.0;
    if (t.active) {
        const uint32_t bits = lane_bits_from_lds<VEC>(sbits, t, nblk, 0u) ^ lane_bits_from_lds<VEC>(sbits + nblk * 4u, t, nblk, 0u);
        uint32_t am[NW];   // both flips on a, as XOR masks of its raw dwords
        {
            const uint32_t W = sign_word<DT, VEC>(bits);
#pragma unroll
            for (int j = 0; j < NW; ++j) am[j] = flip_mask<DT, VEC>(W, j);
        }
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (r + t.WY * u < t.row_end) {
                float x[VEC], y[VEC];
                uint32_t fa[NW];
#pragma unroll
                for (int j = 0; j < NW; ++j) fa[j] = ra[u][j] ^ am[j];
                widen<DT, VEC>(fa, x);
                widen<DT, VEC>(rb[u], y);
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    // A product of two binary32 values is exact in binary64, so the fused form rounds
                    // exactly as a multiplication followed by an addition would: one instruction, same bits.
                    const double xa = (double)x[j], yb = (double)y[j];
                    s_ab = __builtin_fma(xa, yb, s_ab);
                    s_aa = __builtin_fma(xa, xa, s_aa);
                    s_bb = __builtin_fma(yb, yb, s_bb);
                }
            }
    }
    // lanes -> wave (fixed butterfly), waves -> workgroup (fixed order)
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        s_ab += __shfl_down(s_ab, off, 64);
        s_aa += __shfl_down(s_aa, off, 64);
        s_bb += __shfl_down(s_bb, off, 64);
    }
    const uint32_t wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63u) == 0) { swave[wave][0] = s_ab; swave[wave][1] = s_aa; swave[wave][2] = s_bb; }
    __syncthreads();
    if (threadIdx.x < 3) {
        double v = 0.0;
        for (int w = 0; w < WAVES; ++w) v += swave[w][threadIdx.x];
        A.partials[((size_t)A.partial_base + t.id) * 3u + threadIdx.x] = v;
    }
}

// One workgroup: thread q sums partials q, q + 256, ... in order; then a fixed tree over the 256.
__global__ void __launch_bounds__(WG) stats_finalize_kernel(const double *partials, uint32_t n_partials, double *out3)
{
    __shared__ double sh[WG][3];
    double v[3] = {0.0, 0.0, 0.0};
    for (uint32_t q = threadIdx.x; q < n_partials; q += WG)
        for (int c = 0; c < 3; ++c) v[c] += partials[(size_t)q * 3u + c];
    for (int c = 0; c < 3; ++c) sh[threadIdx.x][c] = v[c];
    __syncthreads();
    for (uint32_t half = WG / 2; half > 0; half >>= 1) {
        if (threadIdx.x < half)
            for (int c = 0; c < 3; ++c) sh[threadIdx.x][c] += sh[threadIdx.x + half][c];
        __syncthreads();
    }
    if (threadIdx.x < 3) out3[threadIdx.x] = sh[0][threadIdx.x];
}

// One byte per column: 1 where D is -1.  The bits take the road they take in the streaming kernels:
// the workgroup stages the generator blocks of its "tile" in LDS and every lane picks its bit out of
// them.  Tiles are 192 columns wide, so every other one starts in the middle of a 128-column block.
constexpr uint32_t MASK_TILE_COLS = 192;
__global__ void __launch_bounds__(WG) sign_mask_kernel(uint32_t key_lo, uint32_t key_hi, uint32_t layer,
                                                       int64_t cols, uint8_t *mask_out)
{
    __shared__ uint32_t sbits[3 * 4];   // at most 3 blocks cover 192 columns
    Tile t{};
    t.L.flip = 1u;
    t.L.layer_id = layer;
    t.L.sign_blocks = 0u;
    t.tile_col0 = blockIdx.x * MASK_TILE_COLS;
    t.cw = MASK_TILE_COLS;
    t.col_in_tile = threadIdx.x;
    const uint32_t nblk = stage_sign_bits(sbits, t, nullptr, 1u, key_lo, key_hi);
    __syncthreads();
    const int64_t c = (int64_t)t.tile_col0 + threadIdx.x;
    if (threadIdx.x >= MASK_TILE_COLS || c >= cols) return;
    mask_out[c] = (uint8_t)lane_bits_from_lds<1>(sbits, t, nblk, 0u);
}

// ---------------------------------------------------------------------------
// Bandwidth probe: the same burst shape with nothing of the method in it (no signs, no
// permutation, no format conversion): out = sum of K input streams as 32-bit integer adds, or no
// store at all.  It measures what plain streaming reaches on the machine at hand, which is the
// yardstick the merge (K reads + 1 write) and retrieve (2 reads + 1 write) kernels are held to.
// ---------------------------------------------------------------------------
struct ProbeArgs {
    gcptr in[8];
    gptr out;
    uint64_t n_vec;   // 16-byte vectors per stream
};

template <int K, bool WRITE>
__global__ void __launch_bounds__(WG) probe_kernel(const ProbeArgs P)
{
    constexpr int R = 4;
    // same XCD-contiguous order as the method's kernels (see locate())
    const uint32_t per_xcd = gridDim.x / N_XCD;
    const uint32_t chunk = (blockIdx.x % N_XCD) * per_xcd + blockIdx.x / N_XCD;
    if ((uint64_t)chunk * R * WG >= P.n_vec) return;
    const uint64_t base = ((uint64_t)chunk * R * WG + threadIdx.x) * 16u;
    u32x4 v[R][K];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int k = 0; k < K; ++k)
            v[r][k] = __builtin_nontemporal_load((const RANDES_GLOBAL u32x4 *)(P.in[k] + base + (uint64_t)r * WG * 16u));
    u32x4 res[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        res[r] = v[r][0];
#pragma unroll
        for (int k = 1; k < K; ++k) res[r] += v[r][k];
    }
    load_store_fence();
    if constexpr (WRITE) {
#pragma unroll
        for (int r = 0; r < R; ++r)
            __builtin_nontemporal_store(res[r], (RANDES_GLOBAL u32x4 *)(P.out + base + (uint64_t)r * WG * 16u));
    } else {
        u32x4 t = res[0];
#pragma unroll
        for (int r = 1; r < R; ++r) t ^= res[r];
        // never true for the probe's inputs; keeps the loads alive without a store stream
        if (t.x == 0x9e3779b9u && t.y == 0x7f4a7c15u && t.z == 0xf39cc060u && t.w == 0x5cedc834u)
            __builtin_nontemporal_store(t, (RANDES_GLOBAL u32x4 *)P.out);
    }
}

hipError_t launch_probe(const void *const *inputs, int n_inputs, void *output, uint64_t bytes, int write, hipStream_t s)
{
    ProbeArgs P;
    for (int k = 0; k < 8; ++k) P.in[k] = (gcptr)inputs[k < n_inputs ? k : 0];
    P.out = (gptr)output;
    P.n_vec = bytes / 16u;
    const dim3 grid(xcd_grid((uint32_t)(bytes / PROBE_CHUNK_BYTES))), block(WG);
#define RANDES_PROBE(K) case K: if (write) hipLaunchKernelGGL((probe_kernel<K, true>), grid, block, 0, s, P); \
                                else hipLaunchKernelGGL((probe_kernel<K, false>), grid, block, 0, s, P); break;
    switch (n_inputs) {
    RANDES_PROBE(1) RANDES_PROBE(2) RANDES_PROBE(3) RANDES_PROBE(4)
    RANDES_PROBE(5) RANDES_PROBE(6) RANDES_PROBE(7) RANDES_PROBE(8)
    default: return hipErrorInvalidValue;
    }
#undef RANDES_PROBE
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
// LDS for the staged sign bits: 16 bytes per (task, 128-column generator block of the widest tile,
// plus one block for a tile that starts mid-block).
static size_t sign_bits_lds_bytes(int n_tasks, int vec)
{
    return (size_t)n_tasks * (((size_t)WAVES * 64 * vec + 127) / 128 + 1) * 16;
}

int merge_vec(int dt_in) { return dt_in == DT_BF16 ? 8 : 4; }
int merge_burst_rows() { return MERGE_R; }
int merge_weights_burst_rows() { return MERGE_WEIGHTS_R; }
int retrieve_vec(int dt_merged, int dt_base) { return (dt_merged == DT_BF16 || dt_base == DT_BF16) ? 8 : 4; }
int update_vec(int dt_merged, int dt_delta) { return (dt_merged == DT_BF16 || dt_delta == DT_BF16) ? 8 : 4; }

template <int DTI, int DTO, int VEC>
static hipError_t merge_dispatch(const StreamArgs &a, hipStream_t s)
{
    const dim3 grid(xcd_grid(a.n_tiles, a.xcd_chunk_shift)), block(WG);
    const size_t lds = std::max<size_t>(sign_bits_lds_bytes(a.n_tasks, VEC), a.lds_floor);
    // the element-wise variant and more than KREG_MAX tasks take the any-count kernel
    if constexpr (VEC == 1) {
        hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 0, MERGE_R, false>), grid, block, lds, s, a);
        return hipGetLastError();
    }
    const int kt = a.n_tasks > KREG_MAX ? 0 : a.n_tasks;
    switch (kt) {
#define RANDES_CASE(K) case K: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, K, MERGE_R, false>), grid, block, lds, s, a); break;
    RANDES_CASE(1) RANDES_CASE(2) RANDES_CASE(3) RANDES_CASE(4)
    RANDES_CASE(5) RANDES_CASE(6) RANDES_CASE(7) RANDES_CASE(8)
#undef RANDES_CASE
    default: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 0, MERGE_R, false>), grid, block, lds, s, a); break;
    }
    return hipGetLastError();
}

// weights in, deltas formed on the fly: twice the streams per task, so half the rows per burst
template <int DTI, int DTO, int VEC>
static hipError_t merge_weights_dispatch(const StreamArgs &a, hipStream_t s)
{
    const dim3 grid(xcd_grid(a.n_tiles, a.xcd_chunk_shift)), block(WG);
    const size_t lds = sign_bits_lds_bytes(a.n_tasks, VEC);
    constexpr int R = MERGE_WEIGHTS_R;
    if constexpr (VEC == 1) {
        hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 0, R, true>), grid, block, lds, s, a);
        return hipGetLastError();
    }
    switch (a.n_tasks) {
    case 2: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 2, R, true>), grid, block, lds, s, a); break;
    case 4: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 4, R, true>), grid, block, lds, s, a); break;
    case 8: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 8, R, true>), grid, block, lds, s, a); break;
    default: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 0, R, true>), grid, block, lds, s, a); break;
    }
    return hipGetLastError();
}

hipError_t launch_merge(const StreamArgs &a, int vec, int dt_in, int dt_out, hipStream_t s)
{
    if (a.n_tiles == 0) return hipSuccess;
    if (vec) {
        if (dt_in == DT_F32 && dt_out == DT_F32) return merge_dispatch<DT_F32, DT_F32, 4>(a, s);
        if (dt_in == DT_F32 && dt_out == DT_BF16) return merge_dispatch<DT_F32, DT_BF16, 4>(a, s);
        if (dt_in == DT_BF16 && dt_out == DT_F32) return merge_dispatch<DT_BF16, DT_F32, 8>(a, s);
        return merge_dispatch<DT_BF16, DT_BF16, 8>(a, s);
    }
    if (dt_in == DT_F32 && dt_out == DT_F32) return merge_dispatch<DT_F32, DT_F32, 1>(a, s);
    if (dt_in == DT_F32 && dt_out == DT_BF16) return merge_dispatch<DT_F32, DT_BF16, 1>(a, s);
    if (dt_in == DT_BF16 && dt_out == DT_F32) return merge_dispatch<DT_BF16, DT_F32, 1>(a, s);
    return merge_dispatch<DT_BF16, DT_BF16, 1>(a, s);
}

hipError_t launch_merge_weights(const StreamArgs &a, int vec, int dt_in, int dt_out, hipStream_t s)
{
    if (a.n_tiles == 0) return hipSuccess;
    if (vec) {
        if (dt_in == DT_F32 && dt_out == DT_F32) return merge_weights_dispatch<DT_F32, DT_F32, 4>(a, s);
        if (dt_in == DT_F32 && dt_out == DT_BF16) return merge_weights_dispatch<DT_F32, DT_BF16, 4>(a, s);
        if (dt_in == DT_BF16 && dt_out == DT_F32) return merge_weights_dispatch<DT_BF16, DT_F32, 8>(a, s);
        return merge_weights_dispatch<DT_BF16, DT_BF16, 8>(a, s);
    }
    if (dt_in == DT_F32 && dt_out == DT_F32) return merge_weights_dispatch<DT_F32, DT_F32, 1>(a, s);
    if (dt_in == DT_F32 && dt_out == DT_BF16) return merge_weights_dispatch<DT_F32, DT_BF16, 1>(a, s);
    if (dt_in == DT_BF16 && dt_out == DT_F32) return merge_weights_dispatch<DT_BF16, DT_F32, 1>(a, s);
    return merge_weights_dispatch<DT_BF16, DT_BF16, 1>(a, s);
}

template <int DTM, int DTB, int VEC>
static hipError_t retrieve_dispatch(const StreamArgs &a, int dt_out, hipStream_t s)
{
    const dim3 grid(xcd_grid(a.n_tiles, a.xcd_chunk_shift)), block(WG);
    const size_t lds = std::max<size_t>(sign_bits_lds_bytes(1, VEC), a.lds_floor);
    if (dt_out == DT_F32) hipLaunchKernelGGL((retrieve_kernel<DTM, DTB, DT_F32, VEC>), grid, block, lds, s, a);
    else hipLaunchKernelGGL((retrieve_kernel<DTM, DTB, DT_BF16, VEC>), grid, block, lds, s, a);
    return hipGetLastError();
}

hipError_t launch_retrieve(const StreamArgs &a, int vec, int dt_merged, int dt_base, int dt_out, hipStream_t s)
{
    if (a.n_tiles == 0) return hipSuccess;
    const int sel = (vec ? 4 : 0) | (dt_merged == DT_BF16 ? 2 : 0) | (dt_base == DT_BF16 ? 1 : 0);
    switch (sel) {
    case 0: return retrieve_dispatch<DT_F32, DT_F32, 1>(a, dt_out, s);
    case 1: return retrieve_dispatch<DT_F32, DT_BF16, 1>(a, dt_out, s);
    case 2: return retrieve_dispatch<DT_BF16, DT_F32, 1>(a, dt_out, s);
    case 3: return retrieve_dispatch<DT_BF16, DT_BF16, 1>(a, dt_out, s);
    case 4: return retrieve_dispatch<DT_F32, DT_F32, 4>(a, dt_out, s);
    case 5: return retrieve_dispatch<DT_F32, DT_BF16, 8>(a, dt_out, s);
    case 6: return retrieve_dispatch<DT_BF16, DT_F32, 8>(a, dt_out, s);
    default: return retrieve_dispatch<DT_BF16, DT_BF16, 8>(a, dt_out, s);
    }
}

template <int DT, int VEC>
static hipError_t retrieve_many_dispatch(const StreamArgs &a, hipStream_t s)
{
    const dim3 grid(xcd_grid(a.n_tiles, a.xcd_chunk_shift)), block(WG);
    const size_t lds = sign_bits_lds_bytes(a.n_tasks, VEC);
    switch (a.n_tasks) {
    case 2: hipLaunchKernelGGL((retrieve_many_kernel<DT, VEC, 2>), grid, block, lds, s, a); break;
    case 4: hipLaunchKernelGGL((retrieve_many_kernel<DT, VEC, 4>), grid, block, lds, s, a); break;
    case 8: hipLaunchKernelGGL((retrieve_many_kernel<DT, VEC, 8>), grid, block, lds, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// n_tasks of the arguments = models per pass (2, 4 or 8); one storage type for all three stacks.
hipError_t launch_retrieve_many(const StreamArgs &a, int dt, hipStream_t s)
{
    if (a.n_tiles == 0) return hipSuccess;
    if (dt == DT_F32) return retrieve_many_dispatch<DT_F32, 4>(a, s);
    return retrieve_many_dispatch<DT_BF16, 8>(a, s);
}

template <int DTM, int DTD, int VEC>
static hipError_t update_dispatch(const StreamArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL((update_kernel<DTM, DTD, VEC>), dim3(xcd_grid(a.n_tiles, a.xcd_chunk_shift)), dim3(WG),
                       std::max<size_t>(sign_bits_lds_bytes(1, VEC), a.lds_floor), s, a);
    return hipGetLastError();
}

hipError_t launch_update(const StreamArgs &a, int vec, int dt_merged, int dt_delta, hipStream_t s)
{
    if (a.n_tiles == 0) return hipSuccess;
    const int sel = (vec ? 4 : 0) | (dt_merged == DT_BF16 ? 2 : 0) | (dt_delta == DT_BF16 ? 1 : 0);
    switch (sel) {
    case 0: return update_dispatch<DT_F32, DT_F32, 1>(a, s);
    case 1: return update_dispatch<DT_F32, DT_BF16, 1>(a, s);
    case 2: return update_dispatch<DT_BF16, DT_F32, 1>(a, s);
    case 3: return update_dispatch<DT_BF16, DT_BF16, 1>(a, s);
    case 4: return update_dispatch<DT_F32, DT_F32, 4>(a, s);
    case 5: return update_dispatch<DT_F32, DT_BF16, 8>(a, s);
    case 6: return update_dispatch<DT_BF16, DT_F32, 8>(a, s);
    default: return update_dispatch<DT_BF16, DT_BF16, 8>(a, s);
    }
}

int stats_vec(int dt) { return dt == DT_BF16 ? 8 : 4; }

hipError_t launch_stats(const StreamArgs &a, int vec, int dt, hipStream_t s)
{
    if (a.n_tiles == 0) return hipSuccess;
    const dim3 grid(xcd_grid(a.n_tiles, a.xcd_chunk_shift)), block(WG);
    const size_t lds = 2 * sign_bits_lds_bytes(1, vec ? stats_vec(dt) : 1);
    if (vec) {
        if (dt == DT_F32) hipLaunchKernelGGL((stats_kernel<DT_F32, 4>), grid, block, lds, s, a);
        else hipLaunchKernelGGL((stats_kernel<DT_BF16, 8>), grid, block, lds, s, a);
    } else {
        if (dt == DT_F32) hipLaunchKernelGGL((stats_kernel<DT_F32, 1>), grid, block, lds, s, a);
        else hipLaunchKernelGGL((stats_kernel<DT_BF16, 1>), grid, block, lds, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_stats_finalize(const double *partials, uint32_t n_partials, double *out3, hipStream_t s)
{
    hipLaunchKernelGGL(stats_finalize_kernel, dim3(1), dim3(WG), 0, s, partials, n_partials, out3);
    return hipGetLastError();
}

hipError_t launch_sign_mask(uint32_t key_lo, uint32_t key_hi, uint32_t layer, int64_t cols,
                            uint8_t *mask_out, hipStream_t s)
{
    const uint32_t blocks = (uint32_t)((cols + MASK_TILE_COLS - 1) / MASK_TILE_COLS);
    hipLaunchKernelGGL(sign_mask_kernel, dim3(blocks), dim3(WG), 0, s, key_lo, key_hi, layer, cols, mask_out);
    return hipGetLastError();
}

}  // namespace randes
