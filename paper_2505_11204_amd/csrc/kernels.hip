// gfx950 kernels of the RanDeS hot path: streaming merge (compress), fused
// retrieve, in-place hot-swap update, sign-mask dump, and the MFMA LoRA
// materialiser.  Wavefronts are 64 lanes; a workgroup is 4 waves.
//
// Streaming kernels: one workgroup owns a tile = (slot layer, chunk of rows,
// block of columns).  A lane owns VEC adjacent columns and walks down the rows
// of the tile, so the sign bits of its columns (Sec. 4.4: D is diagonal over the
// columns) are generated once per tile and kept in registers as XOR masks; the
// weight stream itself goes HBM -> registers -> HBM with 16-byte accesses and
// never touches LDS.  The shuffle (Sec. 4.3) costs nothing here: it is already
// folded into the pointer tables.
#include <hip/hip_runtime.h>

#include "launch.hpp"
#include "philox.hpp"

namespace randes {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int WG = 256;          // threads per workgroup
constexpr int WAVES = WG / 64;
constexpr int KREG_MAX = 8;      // merge: up to this many tasks keep their masks in registers
constexpr int MERGE_U = 2;       // merge: rows in flight per wave
constexpr int RETR_U = 4;        // retrieve / update: rows in flight per wave

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// binary32 -> bf16 bits, round to nearest, ties to even; NaN stays quiet NaN.
__device__ __forceinline__ uint32_t bf16_rne(float f)
{
    const uint32_t u = f2u(f);
    uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
    if ((u & 0x7fffffffu) > 0x7f800000u) r = (u >> 16) | 0x40u;
    return r;
}

template <int DT, int VEC> struct NumWords {
    static constexpr int value = (DT == DT_F32) ? VEC : (VEC == 1 ? 1 : VEC / 2);
};

// Load VEC elements of dtype DT from byte address p as raw dwords (bf16 stays packed).
template <int DT, int VEC>
__device__ __forceinline__ void load_raw(const char *p, uint32_t (&raw)[NumWords<DT, VEC>::value])
{
    constexpr int NW = NumWords<DT, VEC>::value;
    if constexpr (NW == 1) {
        if constexpr (DT == DT_F32) raw[0] = __builtin_nontemporal_load((const uint32_t *)p);
        else raw[0] = (uint32_t)__builtin_nontemporal_load((const uint16_t *)p);
    } else if constexpr (NW == 2) {
        const u32x2 q = __builtin_nontemporal_load((const u32x2 *)p);
        raw[0] = q.x; raw[1] = q.y;
    } else {
#pragma unroll
        for (int h = 0; h < NW / 4; ++h) {
            const u32x4 q = __builtin_nontemporal_load((const u32x4 *)p + h);
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

// Store VEC binary32 values as dtype DT at byte address p.
template <int DT, int VEC>
__device__ __forceinline__ void store_vec(char *p, const float (&v)[VEC])
{
    if constexpr (DT == DT_F32) {
        if constexpr (VEC == 1) {
            __builtin_nontemporal_store(v[0], (float *)p);
        } else {
#pragma unroll
            for (int h = 0; h < VEC / 4; ++h) {
                u32x4 q;
                q.x = f2u(v[4 * h]); q.y = f2u(v[4 * h + 1]); q.z = f2u(v[4 * h + 2]); q.w = f2u(v[4 * h + 3]);
                __builtin_nontemporal_store(q, (u32x4 *)p + h);
            }
        }
    } else {
        if constexpr (VEC == 1) {
            __builtin_nontemporal_store((uint16_t)bf16_rne(v[0]), (uint16_t *)p);
        } else if constexpr (VEC == 4) {
            u32x2 q;
            q.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
            q.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
            __builtin_nontemporal_store(q, (u32x2 *)p);
        } else {
            u32x4 q;
            q.x = bf16_rne(v[0]) | (bf16_rne(v[1]) << 16);
            q.y = bf16_rne(v[2]) | (bf16_rne(v[3]) << 16);
            q.z = bf16_rne(v[4]) | (bf16_rne(v[5]) << 16);
            q.w = bf16_rne(v[6]) | (bf16_rne(v[7]) << 16);
            __builtin_nontemporal_store(q, (u32x4 *)p);
        }
    }
}

// Sign bits of columns [col, col + VEC) of one (model, slot layer): bit j set
// means D is -1 at column col + j.  col is a multiple of VEC and VEC divides 32.
template <int VEC>
__device__ __forceinline__ uint32_t lane_sign_bits(uint32_t key_lo, uint32_t key_hi, uint32_t layer, uint32_t col)
{
    const u32x4_t o = sign_block(key_lo, key_hi, layer, col >> 7);
    const uint32_t sel = (col >> 5) & 3u;
    const uint32_t word = sel == 0 ? o.w[0] : sel == 1 ? o.w[1] : sel == 2 ? o.w[2] : o.w[3];
    return (word >> (col & 31u)) & ((VEC == 32) ? 0xffffffffu : ((1u << VEC) - 1u));
}

// Sign bits -> XOR masks laid over the raw dwords of a VEC-element load.
template <int DT, int VEC>
__device__ __forceinline__ void packed_sign_masks(uint32_t bits, uint32_t (&pm)[NumWords<DT, VEC>::value])
{
    if constexpr (DT == DT_F32) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) pm[j] = ((bits >> j) & 1u) << 31;
    } else if constexpr (VEC == 1) {
        pm[0] = (bits & 1u) << 15;
    } else {
#pragma unroll
        for (int j = 0; j < VEC / 2; ++j)
            pm[j] = (((bits >> (2 * j)) & 1u) << 15) | (((bits >> (2 * j + 1)) & 1u) << 31);
    }
}

// acc[j] += (+/-) x[j] for the VEC elements of one task's load; the sign flip is
// an XOR on the packed data, the addition is a plain binary32 add.
template <int DT, int VEC>
__device__ __forceinline__ void accumulate(const uint32_t (&raw)[NumWords<DT, VEC>::value],
                                           const uint32_t (&pm)[NumWords<DT, VEC>::value], float (&acc)[VEC])
{
    constexpr int NW = NumWords<DT, VEC>::value;
    uint32_t t[NW];
#pragma unroll
    for (int j = 0; j < NW; ++j) t[j] = raw[j] ^ pm[j];
    float v[VEC];
    widen<DT, VEC>(t, v);
#pragma unroll
    for (int j = 0; j < VEC; ++j) acc[j] = acc[j] + v[j];
}

// Where this workgroup works.
struct Tile {
    LayerDev L;
    int layer_slot;     // index into the sub-plan's layer array
    uint32_t col;       // first column of this lane
    uint32_t col_in_tile;
    uint32_t row0, row_end;
    uint32_t wy, WY;    // this wave's row phase and the row stride between its rows
    bool active;        // lane has columns inside the layer
};

template <int VEC>
__device__ __forceinline__ Tile locate(const StreamArgs &A)
{
    const uint32_t bid = blockIdx.x;
    int lo = 0, hi = A.n_layers;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (A.tile_begin[mid] <= bid) lo = mid; else hi = mid;
    }
    Tile t;
    t.layer_slot = lo;
    t.L = A.layers[lo];
    const uint32_t idx = bid - A.tile_begin[lo];
    const uint32_t cb = idx % t.L.n_cb, rc = idx / t.L.n_cb;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wx = wave & (t.L.wx - 1u);
    t.WY = (uint32_t)WAVES >> t.L.wx_shift;
    t.wy = wave >> t.L.wx_shift;
    const uint32_t cw = t.L.wx * 64u * VEC;
    t.col_in_tile = (wx * 64u + lane) * VEC;
    t.col = cb * cw + t.col_in_tile;
    t.active = t.col < (uint32_t)t.L.cols;
    t.row0 = rc * t.L.tile_rows;
    const uint32_t re = t.row0 + t.L.tile_rows;
    t.row_end = re < (uint32_t)t.L.rows ? re : (uint32_t)t.L.rows;
    return t;
}

// ---------------------------------------------------------------------------
// compress: merged[l] = sum_i D_i^l-flipped delta_i[src_i(l)], binary32, task order.
// KT > 0: exactly KT tasks, masks hoisted into registers.
// KT = 0: any number of tasks; the tile's sign bits are produced cooperatively
//         into LDS once (bits only: the weight stream still bypasses LDS).
// ---------------------------------------------------------------------------
template <int DTI, int DTO, int VEC, int KT>
__global__ void __launch_bounds__(WG) merge_kernel(const StreamArgs A)
{
    constexpr int NW = NumWords<DTI, VEC>::value;
    constexpr uint32_t EBI = (DTI == DT_F32) ? 4 : 2, EBO = (DTO == DT_F32) ? 4 : 2;
    const Tile t = locate<VEC>(A);
    const uint32_t rb_in = (uint32_t)t.L.cols * EBI, rb_out = (uint32_t)t.L.cols * EBO;
    const size_t tile_in = (size_t)t.row0 * rb_in, tile_out = (size_t)t.row0 * rb_out;
    uint32_t off_in = t.wy * rb_in + t.col * EBI;
    uint32_t off_out = t.wy * rb_out + t.col * EBO;
    const uint32_t step_in = t.WY * rb_in, step_out = t.WY * rb_out;
    char *const dst = (char *)t.L.dst + tile_out;

    if constexpr (KT > 0) {
        if (!t.active) return;
        const char *src[KT];
        uint32_t pm[KT][NW];
#pragma unroll
        for (int i = 0; i < KT; ++i) {
            src[i] = (const char *)A.srcs[(size_t)t.layer_slot * KT + i] + tile_in;
            const uint32_t bits = t.L.flip ? lane_sign_bits<VEC>(A.keys[2 * i], A.keys[2 * i + 1], t.L.layer_id, t.col) : 0u;
            packed_sign_masks<DTI, VEC>(bits, pm[i]);
        }
        uint32_t r = t.row0 + t.wy;
        for (; r + t.WY * (MERGE_U - 1) < t.row_end; r += t.WY * MERGE_U) {
            uint32_t raw[MERGE_U][KT][NW];
#pragma unroll
            for (int u = 0; u < MERGE_U; ++u)
#pragma unroll
                for (int i = 0; i < KT; ++i) load_raw<DTI, VEC>(src[i] + off_in + u * step_in, raw[u][i]);
#pragma unroll
            for (int u = 0; u < MERGE_U; ++u) {
                float acc[VEC];
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[j] = 0.0f;
#pragma unroll
                for (int i = 0; i < KT; ++i) accumulate<DTI, VEC>(raw[u][i], pm[i], acc);
                store_vec<DTO, VEC>(dst + off_out + u * step_out, acc);
            }
            off_in += MERGE_U * step_in;
            off_out += MERGE_U * step_out;
        }
        for (; r < t.row_end; r += t.WY) {
            uint32_t raw[KT][NW];
#pragma unroll
            for (int i = 0; i < KT; ++i) load_raw<DTI, VEC>(src[i] + off_in, raw[i]);
            float acc[VEC];
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc[j] = 0.0f;
#pragma unroll
            for (int i = 0; i < KT; ++i) accumulate<DTI, VEC>(raw[i], pm[i], acc);
            store_vec<DTO, VEC>(dst + off_out, acc);
            off_in += step_in;
            off_out += step_out;
        }
    } else {
        extern __shared__ uint32_t sbits[];                 // [n_tasks][words per tile row]
        __shared__ const char *sptr[RANDES_MAX_TASKS];      // tile base pointer of every task
        const uint32_t cw = t.L.wx * 64u * VEC;             // columns of the workgroup's tile
        const uint32_t K = (uint32_t)A.n_tasks;
        // The tile's first column is a multiple of cw, and cw is a multiple of 64, so a tile may
        // start in the middle of a 128-column generator block: bits are stored relative to
        // the block that contains the tile's first column.
        const uint32_t tile_col0 = t.col - t.col_in_tile;
        const uint32_t lead = tile_col0 & 127u;             // columns of the first block before the tile
        const uint32_t nblk = (lead + cw + 127u) / 128u;    // generator blocks per task
        for (uint32_t q = threadIdx.x; q < K * nblk; q += WG) {
            const uint32_t i = q / nblk, blk = q % nblk;
            u32x4_t o;
            if (t.L.flip) o = sign_block(A.keys[2 * i], A.keys[2 * i + 1], t.L.layer_id, (tile_col0 >> 7) + blk);
            else { o.w[0] = o.w[1] = o.w[2] = o.w[3] = 0u; }
            uint32_t *w = sbits + ((size_t)i * nblk + blk) * 4u;
            w[0] = o.w[0]; w[1] = o.w[1]; w[2] = o.w[2]; w[3] = o.w[3];
        }
        for (uint32_t i = threadIdx.x; i < K; i += WG)
            sptr[i] = (const char *)A.srcs[(size_t)t.layer_slot * K + i] + tile_in;
        __syncthreads();
        if (!t.active) return;
        const uint32_t rel = lead + t.col_in_tile;          // column relative to the first stored block
        const uint32_t widx = rel >> 5, sh = rel & 31u;
        constexpr uint32_t vm = (VEC == 32) ? 0xffffffffu : ((1u << VEC) - 1u);
        constexpr int KC = 8;
        uint32_t r = t.row0 + t.wy;
        for (; r < t.row_end; r += t.WY * MERGE_U) {
            const bool two = (r + t.WY) < t.row_end;   // MERGE_U == 2 rows per step, second may be missing
            float acc[MERGE_U][VEC];
#pragma unroll
            for (int u = 0; u < MERGE_U; ++u)
#pragma unroll
                for (int j = 0; j < VEC; ++j) acc[u][j] = 0.0f;
            for (uint32_t i0 = 0; i0 < K; i0 += KC) {
                uint32_t raw[MERGE_U][KC][NW];
#pragma unroll
                for (int j = 0; j < KC; ++j) {
                    if (i0 + j < K) {
                        const char *p = sptr[i0 + j] + off_in;
                        load_raw<DTI, VEC>(p, raw[0][j]);
                        if (two) load_raw<DTI, VEC>(p + step_in, raw[1][j]);
                    }
                }
#pragma unroll
                for (int j = 0; j < KC; ++j) {
                    if (i0 + j < K) {
                        const uint32_t bits = (sbits[(size_t)(i0 + j) * nblk * 4u + widx] >> sh) & vm;
                        uint32_t pm[NW];
                        packed_sign_masks<DTI, VEC>(bits, pm);
                        accumulate<DTI, VEC>(raw[0][j], pm, acc[0]);
                        if (two) accumulate<DTI, VEC>(raw[1][j], pm, acc[1]);
                    }
                }
            }
            store_vec<DTO, VEC>(dst + off_out, acc[0]);
            if (two) store_vec<DTO, VEC>(dst + off_out + step_out, acc[1]);
            off_in += MERGE_U * step_in;
            off_out += MERGE_U * step_out;
        }
    }
}

// ---------------------------------------------------------------------------
// retrieve: out[t] = fma(lambda, D-flipped merged[l], base[t]), t = src(l).
// ---------------------------------------------------------------------------
template <int DTM, int DTB, int DTO, int VEC>
__global__ void __launch_bounds__(WG) retrieve_kernel(const StreamArgs A)
{
    constexpr uint32_t EBM = (DTM == DT_F32) ? 4 : 2, EBB = (DTB == DT_F32) ? 4 : 2, EBO = (DTO == DT_F32) ? 4 : 2;
    const Tile t = locate<VEC>(A);
    if (!t.active) return;
    const uint32_t cols = (uint32_t)t.L.cols;
    const char *pm_ = (const char *)t.L.a + (size_t)t.row0 * cols * EBM;
    const char *pb_ = (const char *)t.L.b + (size_t)t.row0 * cols * EBB;
    char *po_ = (char *)t.L.dst + (size_t)t.row0 * cols * EBO;
    const uint32_t bits = t.L.flip ? lane_sign_bits<VEC>(A.key_lo, A.key_hi, t.L.layer_id, t.col) : 0u;
    uint32_t sm[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) sm[j] = ((bits >> j) & 1u) << 31;
    const float lambda = A.lambda;
    uint32_t e = t.wy * cols + t.col;               // element offset inside the tile
    const uint32_t estep = t.WY * cols;
    uint32_t r = t.row0 + t.wy;
    for (; r + t.WY * (RETR_U - 1) < t.row_end; r += t.WY * RETR_U) {
        uint32_t rm[RETR_U][NumWords<DTM, VEC>::value], rb[RETR_U][NumWords<DTB, VEC>::value];
#pragma unroll
        for (int u = 0; u < RETR_U; ++u) {
            load_raw<DTM, VEC>(pm_ + (size_t)(e + u * estep) * EBM, rm[u]);
            load_raw<DTB, VEC>(pb_ + (size_t)(e + u * estep) * EBB, rb[u]);
        }
#pragma unroll
        for (int u = 0; u < RETR_U; ++u) {
            float m[VEC], b[VEC], o[VEC];
            widen<DTM, VEC>(rm[u], m);
            widen<DTB, VEC>(rb[u], b);
#pragma unroll
            for (int j = 0; j < VEC; ++j) o[j] = __builtin_fmaf(lambda, u2f(f2u(m[j]) ^ sm[j]), b[j]);
            store_vec<DTO, VEC>(po_ + (size_t)(e + u * estep) * EBO, o);
        }
        e += RETR_U * estep;
    }
    for (; r < t.row_end; r += t.WY) {
        uint32_t rm[NumWords<DTM, VEC>::value], rb[NumWords<DTB, VEC>::value];
        load_raw<DTM, VEC>(pm_ + (size_t)e * EBM, rm);
        load_raw<DTB, VEC>(pb_ + (size_t)e * EBB, rb);
        float m[VEC], b[VEC], o[VEC];
        widen<DTM, VEC>(rm, m);
        widen<DTB, VEC>(rb, b);
#pragma unroll
        for (int j = 0; j < VEC; ++j) o[j] = __builtin_fmaf(lambda, u2f(f2u(m[j]) ^ sm[j]), b[j]);
        store_vec<DTO, VEC>(po_ + (size_t)e * EBO, o);
        e += estep;
    }
}

// ---------------------------------------------------------------------------
// hot swap: merged[l] <- merged[l] +/- D-flipped delta[src(l)].
// ---------------------------------------------------------------------------
template <int DTM, int DTD, int VEC>
__global__ void __launch_bounds__(WG) update_kernel(const StreamArgs A)
{
    constexpr uint32_t EBM = (DTM == DT_F32) ? 4 : 2, EBD = (DTD == DT_F32) ? 4 : 2;
    const Tile t = locate<VEC>(A);
    if (!t.active) return;
    const uint32_t cols = (uint32_t)t.L.cols;
    char *pm_ = (char *)t.L.dst + (size_t)t.row0 * cols * EBM;
    const char *pd_ = (const char *)t.L.a + (size_t)t.row0 * cols * EBD;
    uint32_t bits = t.L.flip ? lane_sign_bits<VEC>(A.key_lo, A.key_hi, t.L.layer_id, t.col) : 0u;
    if (A.negate) bits = ~bits;
    uint32_t sm[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) sm[j] = ((bits >> j) & 1u) << 31;
    uint32_t e = t.wy * cols + t.col;
    const uint32_t estep = t.WY * cols;
    for (uint32_t r = t.row0 + t.wy; r < t.row_end; r += t.WY) {
        uint32_t rm[NumWords<DTM, VEC>::value], rd[NumWords<DTD, VEC>::value];
        load_raw<DTM, VEC>(pm_ + (size_t)e * EBM, rm);
        load_raw<DTD, VEC>(pd_ + (size_t)e * EBD, rd);
        float m[VEC], d[VEC], o[VEC];
        widen<DTM, VEC>(rm, m);
        widen<DTD, VEC>(rd, d);
#pragma unroll
        for (int j = 0; j < VEC; ++j) o[j] = m[j] + u2f(f2u(d[j]) ^ sm[j]);
        store_vec<DTM, VEC>(pm_ + (size_t)e * EBM, o);
        e += estep;
    }
}

// One byte per column: 1 where D is -1.
__global__ void __launch_bounds__(WG) sign_mask_kernel(uint32_t key_lo, uint32_t key_hi, uint32_t layer,
                                                       int64_t cols, uint8_t *mask_out)
{
    const int64_t c = (int64_t)blockIdx.x * WG + threadIdx.x;
    if (c >= cols) return;
    mask_out[c] = (uint8_t)lane_sign_bits<1>(key_lo, key_hi, layer, (uint32_t)c);
}

// ---------------------------------------------------------------------------
// LoRA delta on the matrix cores: out = scale * B (rows x rank) * A (rank x cols).
// A workgroup owns 32 rows x 128 columns; each wave owns one 32 x 32 block and
// runs v_mfma_f32_32x32x16_bf16 (bf16 factors) or v_mfma_f32_32x32x2_f32 over
// the rank.  Operand layout of the 32x32 MFMAs: lane L supplies row (L % 32) of
// the left operand and column (L % 32) of the right operand, for the depth
// slice owned by lane half (L / 32); accumulator register v of lane L is
// output row 8*(v/4) + 4*(L/32) + (v%4), column L % 32.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

template <int DTAB, int DTO>
__global__ void __launch_bounds__(WG) lora_kernel(const LoraItem *items, int32_t n_items, int32_t rank, float scale)
{
    const uint32_t bid = blockIdx.x;
    int lo = 0, hi = n_items;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (items[mid].tile_begin <= bid) lo = mid; else hi = mid;
    }
    const LoraItem it = items[lo];
    const uint32_t idx = bid - it.tile_begin;
    const uint32_t tx = idx % it.tiles_x, ty = idx / it.tiles_x;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t half = lane >> 5, l32 = lane & 31u;
    const int64_t row = (int64_t)ty * LORA_TILE_M + l32;            // left operand row of this lane
    const int64_t col = (int64_t)tx * LORA_TILE_N + wave * 32 + l32; // right operand column of this lane
    const bool row_ok = row < it.rows, col_ok = col < it.cols;
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.0f;

    if constexpr (DTAB == DT_BF16) {
        const uint16_t *Bp = (const uint16_t *)it.B;
        const uint16_t *Ap = (const uint16_t *)it.A;
        for (int32_t k0 = 0; k0 < rank; k0 += 16) {
            uint16_t ab[8], bb[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t k = k0 + (int32_t)half * 8 + q;
                const bool k_ok = k < rank;
                ab[q] = (row_ok && k_ok) ? Bp[row * rank + k] : (uint16_t)0;
                bb[q] = (col_ok && k_ok) ? Ap[(int64_t)k * it.cols + col] : (uint16_t)0;
            }
            bf16x8 av, bv;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                av[q] = __builtin_bit_cast(__bf16, ab[q]);
                bv[q] = __builtin_bit_cast(__bf16, bb[q]);
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
        }
    } else {
        const float *Bp = (const float *)it.B;
        const float *Ap = (const float *)it.A;
        for (int32_t k0 = 0; k0 < rank; k0 += 2) {
            const int32_t k = k0 + (int32_t)half;
            const bool k_ok = k < rank;
            const float a = (row_ok && k_ok) ? Bp[row * rank + k] : 0.0f;
            const float b = (col_ok && k_ok) ? Ap[(int64_t)k * it.cols + col] : 0.0f;
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
    }

    if (!col_ok) return;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int64_t orow = (int64_t)ty * LORA_TILE_M + 8 * (v / 4) + 4 * (int)half + (v % 4);
        if (orow < it.rows) {
            const float val = scale * acc[v];
            if constexpr (DTO == DT_F32) ((float *)it.out)[orow * it.cols + col] = val;
            else ((uint16_t *)it.out)[orow * it.cols + col] = (uint16_t)bf16_rne(val);
        }
    }
}

// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
int merge_vec(int dt_in) { return dt_in == DT_BF16 ? 8 : 4; }
int retrieve_vec(int dt_merged, int dt_base) { return (dt_merged == DT_BF16 || dt_base == DT_BF16) ? 8 : 4; }
int update_vec(int dt_merged, int dt_delta) { return (dt_merged == DT_BF16 || dt_delta == DT_BF16) ? 8 : 4; }

template <int DTI, int DTO, int VEC>
static hipError_t merge_dispatch(const StreamArgs &a, hipStream_t s)
{
    const dim3 grid(a.n_tiles), block(WG);
    // element-wise variant always stages bits in LDS; the vector variant does so above KREG_MAX tasks
    const int kt = (VEC == 1 || a.n_tasks > KREG_MAX) ? 0 : a.n_tasks;
    const size_t lds = (size_t)a.n_tasks * (((size_t)WAVES * 64 * VEC + 127) / 128 + 1) * 16;
    switch (kt) {
#define RANDES_CASE(K) case K: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, K>), grid, block, 0, s, a); break;
    RANDES_CASE(1) RANDES_CASE(2) RANDES_CASE(3) RANDES_CASE(4)
    RANDES_CASE(5) RANDES_CASE(6) RANDES_CASE(7) RANDES_CASE(8)
#undef RANDES_CASE
    default: hipLaunchKernelGGL((merge_kernel<DTI, DTO, VEC, 0>), grid, block, lds, s, a); break;
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

template <int DTM, int DTB, int VEC>
static hipError_t retrieve_dispatch(const StreamArgs &a, int dt_out, hipStream_t s)
{
    const dim3 grid(a.n_tiles), block(WG);
    if (dt_out == DT_F32) hipLaunchKernelGGL((retrieve_kernel<DTM, DTB, DT_F32, VEC>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((retrieve_kernel<DTM, DTB, DT_BF16, VEC>), grid, block, 0, s, a);
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

template <int DTM, int DTD, int VEC>
static hipError_t update_dispatch(const StreamArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL((update_kernel<DTM, DTD, VEC>), dim3(a.n_tiles), dim3(WG), 0, s, a);
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

hipError_t launch_sign_mask(uint32_t key_lo, uint32_t key_hi, uint32_t layer, int64_t cols,
                            uint8_t *mask_out, hipStream_t s)
{
    const uint32_t blocks = (uint32_t)((cols + WG - 1) / WG);
    hipLaunchKernelGGL(sign_mask_kernel, dim3(blocks), dim3(WG), 0, s, key_lo, key_hi, layer, cols, mask_out);
    return hipGetLastError();
}

hipError_t launch_lora(const LoraItem *items_dev, int32_t n_items, uint32_t n_tiles, int32_t rank, float scale,
                       int dt_ab, int dt_out, hipStream_t s)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(n_tiles), block(WG);
    if (dt_ab == DT_BF16 && dt_out == DT_BF16)
        hipLaunchKernelGGL((lora_kernel<DT_BF16, DT_BF16>), grid, block, 0, s, items_dev, n_items, rank, scale);
    else if (dt_ab == DT_BF16)
        hipLaunchKernelGGL((lora_kernel<DT_BF16, DT_F32>), grid, block, 0, s, items_dev, n_items, rank, scale);
    else if (dt_out == DT_BF16)
        hipLaunchKernelGGL((lora_kernel<DT_F32, DT_BF16>), grid, block, 0, s, items_dev, n_items, rank, scale);
    else
        hipLaunchKernelGGL((lora_kernel<DT_F32, DT_F32>), grid, block, 0, s, items_dev, n_items, rank, scale);
    return hipGetLastError();
}

}  // namespace randes
