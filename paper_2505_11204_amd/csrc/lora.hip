// LoRA deltas on the matrix cores (Sec. "Parameter Efficient Finetuning (PEFT) Model Compression":
// Theta_i = Theta_0 + lambda L_i with L_i = B_i A_i).
//
//   out = scale * sum over segments s of  B_s (rows x rank) * A_s (rank x cols) * D_s
//
// One segment without a sign flip is the plain materialisation L = scale * B A.  K segments, each
// with the sign diagonal D of its model, is the superposition of K adapters written once:
// sum_i (B_i A_i) D_i = [B_1 .. B_K] [A_1 D_1; ..; A_K D_K], a rank K*r contraction.
//
// A workgroup (4 waves) owns 512 columns and 4 or 8 consecutive blocks of 32 rows; per block
// each wave owns 32 x 128 = four 32x32 MFMA accumulators.  Per 16-deep slice of the depth (segments
// x rank) the workgroup stages A's 16 x 512 slab, sign-flipped, into LDS with 16-byte accesses
// (row-major, as in memory); a lane then gathers the 8 depth values of its column with 2-byte LDS
// reads, which are conflict-free because neighbouring lanes read neighbouring columns.  Up to 8
// slices (one rank-16 adapter, or 8 of them superposed) are staged and gathered once per workgroup
// and kept in registers for all its row blocks; deeper products stage per row block.  B's rows come straight from global memory (16 bytes per lane).  bf16
// results go back through LDS so that every lane stores 16 contiguous bytes.  The kernel is bound
// by the output write.
//
// Operand layout of the 32x32 MFMAs: lane L supplies row (L % 32) of the left operand and column
// (L % 32) of the right operand for the depth slice owned by lane half (L / 32); accumulator
// register v of lane L is row 8*(v/4) + 4*(L/32) + (v%4), column L % 32 of the product.  The
// product is formed transposed (A^T-slice as left operand, B^T as right), so that a lane ends up
// with four adjacent output columns per accumulator quad and can hand them to LDS 8 (bf16) or 16
// (binary32) bytes at a time; rows then leave LDS as 16-byte pieces of contiguous row segments.
#include <hip/hip_runtime.h>

#include "device_util.hpp"
#include "launch.hpp"
#include "philox.hpp"

namespace randes {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Two binary32 values -> one dword of two bf16, with the hardware's packed round-to-nearest-even
// conversion (v_cvt_pk_bf16_f32).  Used only here, where results are checked to a tolerance; the
// streaming kernels use the integer sequence whose every bit the oracle reproduces.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 v;
    v.x = lo; v.y = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

constexpr int KCH = LORA_DEPTH_SLICE;   // rank slice per staging step
constexpr int AS_STRIDE = LORA_TILE_N + 8;   // elements per staged depth row (keeps rows 16-byte aligned)
constexpr int ST_ROW_BYTES = 272;       // staged output row: 128 bf16 or 64 binary32 columns, plus 16 bytes
constexpr int ST_STRIDE = ST_ROW_BYTES / 2;     // in bf16 elements
constexpr int ST_STRIDE_F = ST_ROW_BYTES / 4;   // in binary32 elements
constexpr int LORA_RESIDENT_MAX = 8;    // depth slices whose operand fragments a wave can keep in registers

// Sign bits of the tile's 512 columns for one segment: four generator blocks (tiles start on
// multiples of 512).  Threads 0..3; made visible by the barrier that precedes the staging.
__device__ __forceinline__ void lora_sign_bits(uint32_t *sbits, const LoraSeg &S, int32_t col0, uint32_t tid)
{
    if (tid < LORA_TILE_N / 128) {
        u32x4_t o;
        if (S.flip) o = sign_block(S.key_lo, S.key_hi, S.layer_id, ((uint32_t)col0 >> 7) + tid);
        else { o.w[0] = o.w[1] = o.w[2] = o.w[3] = 0u; }
        sbits[tid * 4 + 0] = o.w[0]; sbits[tid * 4 + 1] = o.w[1];
        sbits[tid * 4 + 2] = o.w[2]; sbits[tid * 4 + 3] = o.w[3];
    }
}

// Stage A[k0 .. k0+15][col0 .. col0+511] of one segment, sign-flipped, row-major into LDS.
template <int DTAB>
__device__ __forceinline__ void lora_stage_slab(char *smem, const uint32_t *sbits, const LoraSeg &S, int32_t k0,
                                                int32_t rank, int32_t col0, int32_t cols, uint32_t tid)
{
    if constexpr (DTAB == DT_BF16) {
        const bool a_vec_ok = (cols % 8 == 0) && (((uintptr_t)S.A & 15u) == 0);
        uint16_t *As = (uint16_t *)smem;
        const RANDES_GLOBAL uint16_t *Ap = (const RANDES_GLOBAL uint16_t *)S.A;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int32_t kk = (int32_t)(tid >> 6) + 4 * p;      // 0..15 inside the slice
            const int32_t k = k0 + kk;
            const int32_t c8 = (int32_t)(tid & 63u) * 8;         // column inside the tile
            const int32_t c = col0 + c8;
            uint32_t w[4] = {0u, 0u, 0u, 0u};
            if (k < rank && c < cols) {
                if (a_vec_ok) {
                    const u32x4 q = *(const RANDES_GLOBAL u32x4 *)(Ap + (int64_t)k * cols + c);
                    w[0] = q.x; w[1] = q.y; w[2] = q.z; w[3] = q.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (c + j < cols) w[j >> 1] |= (uint32_t)Ap[(int64_t)k * cols + c + j] << (16 * (j & 1));
                }
            }
            const uint32_t bits = (sbits[c8 >> 5] >> (c8 & 31)) & 0xffu;
            u32x4 q;
            q.x = w[0] ^ ((((bits >> 0) & 1u) << 15) | (((bits >> 1) & 1u) << 31));
            q.y = w[1] ^ ((((bits >> 2) & 1u) << 15) | (((bits >> 3) & 1u) << 31));
            q.z = w[2] ^ ((((bits >> 4) & 1u) << 15) | (((bits >> 5) & 1u) << 31));
            q.w = w[3] ^ ((((bits >> 6) & 1u) << 15) | (((bits >> 7) & 1u) << 31));
            *(u32x4 *)(As + kk * AS_STRIDE + c8) = q;
        }
    } else {
        uint32_t *As = (uint32_t *)smem;
        const RANDES_GLOBAL uint32_t *Ap = (const RANDES_GLOBAL uint32_t *)S.A;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int32_t kk = (int32_t)(tid >> 7) + 2 * p;      // 0..15
            const int32_t k = k0 + kk;
            const int32_t c4 = (int32_t)(tid & 127u) * 4;
            const int32_t c = col0 + c4;
            const uint32_t bits = (sbits[c4 >> 5] >> (c4 & 31)) & 0xfu;
            u32x4 q = {0u, 0u, 0u, 0u};
            if (k < rank) {
                if (c < cols) q.x = Ap[(int64_t)k * cols + c];
                if (c + 1 < cols) q.y = Ap[(int64_t)k * cols + c + 1];
                if (c + 2 < cols) q.z = Ap[(int64_t)k * cols + c + 2];
                if (c + 3 < cols) q.w = Ap[(int64_t)k * cols + c + 3];
            }
            q.x ^= ((bits >> 0) & 1u) << 31; q.y ^= ((bits >> 1) & 1u) << 31;
            q.z ^= ((bits >> 2) & 1u) << 31; q.w ^= ((bits >> 3) & 1u) << 31;
            *(u32x4 *)(As + kk * AS_STRIDE + c4) = q;
        }
    }
}

// bf16 factors: this lane's operand fragments (8 depth values of one column) of the wave's four
// 32-column blocks, gathered from the staged slab.
__device__ __forceinline__ void lora_gather(const char *smem, uint32_t wave, uint32_t half, uint32_t l32, u32x4 frag[4])
{
    const uint16_t *As = (const uint16_t *)smem;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const uint32_t c = wave * 128u + (uint32_t)b * 32u + l32;
        const uint16_t *col = As + (half * 8u) * AS_STRIDE + c;
        frag[b].x = (uint32_t)col[0 * AS_STRIDE] | ((uint32_t)col[1 * AS_STRIDE] << 16);
        frag[b].y = (uint32_t)col[2 * AS_STRIDE] | ((uint32_t)col[3 * AS_STRIDE] << 16);
        frag[b].z = (uint32_t)col[4 * AS_STRIDE] | ((uint32_t)col[5 * AS_STRIDE] << 16);
        frag[b].w = (uint32_t)col[6 * AS_STRIDE] | ((uint32_t)col[7 * AS_STRIDE] << 16);
    }
}

// bf16 factors: this lane's 8 depth values B[my_row][k0 + 8*half ..] of one segment.
__device__ __forceinline__ u32x4 lora_b_slice(const LoraSeg &S, int32_t my_row, bool row_ok, int32_t k0,
                                              uint32_t half, int32_t rank)
{
    const bool b_vec_ok = (rank % 8 == 0) && (((uintptr_t)S.B & 15u) == 0);
    const RANDES_GLOBAL uint16_t *Bp = (const RANDES_GLOBAL uint16_t *)S.B;
    const int32_t kb = k0 + (int32_t)half * 8;
    u32x4 q = {0u, 0u, 0u, 0u};
    if (row_ok && kb < rank) {
        if (b_vec_ok) {
            q = *(const RANDES_GLOBAL u32x4 *)(Bp + (int64_t)my_row * rank + kb);
        } else {
            uint32_t aw[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j)
                if (kb + j < rank) aw[j >> 1] |= (uint32_t)Bp[(int64_t)my_row * rank + kb + j] << (16 * (j & 1));
            q.x = aw[0]; q.y = aw[1]; q.z = aw[2]; q.w = aw[3];
        }
    }
    return q;
}

// binary32 factors: the 16-deep slice through the 32x32x2 MFMAs, right operand read from the slab.
__device__ __forceinline__ void lora_mma_f32(const char *smem, const LoraSeg &S, int32_t my_row, bool row_ok,
                                             int32_t k0, int32_t rank, uint32_t wave, uint32_t half, uint32_t l32,
                                             f32x16 acc[4])
{
    const float *As = (const float *)smem;
    const RANDES_GLOBAL float *Bp = (const RANDES_GLOBAL float *)S.B;
#pragma unroll
    for (int st = 0; st < KCH / 2; ++st) {
        const int32_t kk = 2 * st + (int32_t)half;
        const int32_t k = k0 + kk;
        const float a = (row_ok && k < rank) ? Bp[(int64_t)my_row * rank + k] : 0.0f;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const uint32_t c = wave * 128u + (uint32_t)b * 32u + l32;
            acc[b] = __builtin_amdgcn_mfma_f32_32x32x2f32(As[kk * AS_STRIDE + c], a, acc[b], 0, 0, 0);
        }
    }
}

// RES > 0: every output matrix has at most RES depth slices (segments x ceil(rank / 16)); the
// workgroup stages each slice once and, for bf16 factors, every wave keeps the gathered fragments
// of all slices in registers, so that its row blocks only load their slices of B and multiply.
// (binary32 factors: RES = 1 only, the single slab stays in LDS.)  RES = 0: any depth, slices
// staged again for every row block.
template <int DTAB, int DTO, int RES>
__global__ void __launch_bounds__(WG) lora_kernel(const LoraItem *items, int32_t n_items, const LoraSeg *segs,
                                                  const uint32_t *coarse, int32_t rank, float scale, int32_t row_tiles)
{
    static_assert(RES >= 0 && RES <= LORA_RESIDENT_MAX && (DTAB == DT_BF16 || RES <= 1), "unsupported residency");
    constexpr int AT_BYTES = KCH * AS_STRIDE * (DTAB == DT_BF16 ? 2 : 4);
    constexpr int ST_BYTES = WAVES * LORA_TILE_M * ST_ROW_BYTES;
    __shared__ __attribute__((aligned(16))) char smem[AT_BYTES];       // the staged slab of A
    __shared__ __attribute__((aligned(16))) char sstage[ST_BYTES];     // output staging, one region per wave
    __shared__ uint32_t sbits[LORA_TILE_N / 32];

    const uint32_t bid = blockIdx.x;
    // coarse[i] = matrix that holds workgroup 64 * i: narrows the search to a step or two
    int lo = (int)coarse[bid >> 6], hi = (int)coarse[(bid >> 6) + 1] + 1;
    if (hi > n_items) hi = n_items;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (items[mid].tile_begin <= bid) lo = mid; else hi = mid;
    }
    const LoraItem it = items[lo];
    const uint32_t idx = bid - it.tile_begin;
    const uint32_t tx = idx % it.tiles_x, ty = idx / it.tiles_x;
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lane = tid & 63u, half = lane >> 5, l32 = lane & 31u;
    const int32_t col0 = (int32_t)tx * LORA_TILE_N;
    const int32_t rows = it.rows, cols = it.cols;
    const int32_t slices_per_seg = (rank + KCH - 1) / KCH;
    const int32_t n_slices = (int32_t)it.n_seg * slices_per_seg;    // <= RES when RES > 0 (host-checked)

    constexpr int NF = RES > 0 ? RES : 1;
    u32x4 frag[NF][4];   // bf16 factors: right-operand fragments per resident slice (RES = 0: of the current slice)
    // Resident variants with registers to spare fetch a row block's slices of B one block ahead
    // (the first block's while the slabs are staged), so that no row block waits for global memory.
    constexpr bool AHEAD = DTAB == DT_BF16 && (RES == 1 || RES == 4);
    constexpr int NB_AHEAD = AHEAD ? RES : 1;
    u32x4 bnext[NB_AHEAD];
    auto fetch_b = [&](int rt, u32x4 *dst) {
        const int32_t r0 = ((int32_t)ty * row_tiles + rt) * LORA_TILE_M;
        const int32_t row = r0 + (int32_t)l32;
#pragma unroll
        for (int s = 0; s < NF; ++s)
            if (s < n_slices)
                dst[s] = lora_b_slice(segs[it.seg_begin + (uint32_t)(s / slices_per_seg)], row, row < rows,
                                      (s % slices_per_seg) * KCH, half, rank);
    };
    if constexpr (AHEAD) fetch_b(0, bnext);
    if constexpr (RES > 0) {
#pragma unroll
        for (int s = 0; s < RES; ++s) {
            if (s < n_slices) {
                const LoraSeg S = segs[it.seg_begin + (uint32_t)(s / slices_per_seg)];
                lora_sign_bits(sbits, S, col0, tid);
                __syncthreads();   // the previous slab is consumed; sbits are visible
                lora_stage_slab<DTAB>(smem, sbits, S, (s % slices_per_seg) * KCH, rank, col0, cols, tid);
                __syncthreads();
                if constexpr (DTAB == DT_BF16) lora_gather(smem, wave, half, l32, frag[s]);
            }
        }
    }

  for (int rt = 0; rt < row_tiles; ++rt) {
    const int32_t row0 = ((int32_t)ty * row_tiles + rt) * LORA_TILE_M;
    if (row0 >= rows) break;
    const int32_t my_row = row0 + (int32_t)l32;              // left-operand row of this lane
    const bool row_ok = my_row < rows;

    f32x16 acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[b][v] = 0.0f;

    if constexpr (RES > 0) {
        if constexpr (DTAB == DT_BF16) {
            u32x4 bsl[RES];   // all loads of the row block go out before the first multiply
            if constexpr (AHEAD) {
#pragma unroll
                for (int s = 0; s < RES; ++s) bsl[s] = bnext[s];
                if (rt + 1 < row_tiles && row0 + LORA_TILE_M < rows) fetch_b(rt + 1, bnext);
            } else {
                fetch_b(rt, bsl);
            }
#pragma unroll
            for (int s = 0; s < RES; ++s)
                if (s < n_slices) {
                    const bf16x8 av = __builtin_bit_cast(bf16x8, bsl[s]);
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, frag[s][b]), av, acc[b], 0, 0, 0);
                }
        } else {
            lora_mma_f32(smem, segs[it.seg_begin], my_row, row_ok, 0, rank, wave, half, l32, acc);
        }
    } else {
        for (uint32_t sg = 0; sg < it.n_seg; ++sg) {
            const LoraSeg S = segs[it.seg_begin + sg];
            lora_sign_bits(sbits, S, col0, tid);
            for (int32_t k0 = 0; k0 < rank; k0 += KCH) {
                // this lane's slice of B: issued first so that it is in flight during the staging
                u32x4 bq = {0u, 0u, 0u, 0u};
                if constexpr (DTAB == DT_BF16) bq = lora_b_slice(S, my_row, row_ok, k0, half, rank);
                __syncthreads();   // the slab of the previous step is consumed; sbits are visible
                lora_stage_slab<DTAB>(smem, sbits, S, k0, rank, col0, cols, tid);
                __syncthreads();
                if constexpr (DTAB == DT_BF16) {
                    lora_gather(smem, wave, half, l32, frag[0]);
                    const bf16x8 av = __builtin_bit_cast(bf16x8, bq);
#pragma unroll
                    for (int b = 0; b < 4; ++b)
                        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, frag[0][b]), av, acc[b], 0, 0, 0);
                } else {
                    lora_mma_f32(smem, S, my_row, row_ok, k0, rank, wave, half, l32, acc);
                }
            }
        }
    }

    // ---- epilogue ----
    // transposed product: this lane holds output row l32, columns b*32 + 8*g + 4*half + (0..3) of
    // its wave's 32 x 128 block in acc[b][4*g .. 4*g+3]
    const int32_t wcol0 = col0 + (int32_t)wave * 128;    // first column of this wave's block
    if constexpr (DTO == DT_F32) {
        // two passes of 64 columns through the wave's staging region
        float *stg = (float *)sstage + wave * (LORA_TILE_M * ST_STRIDE_F);
        RANDES_GLOBAL float *out = (RANDES_GLOBAL float *)it.out;
        const bool o_vec_ok = (cols % 4 == 0) && (((uintptr_t)it.out & 15u) == 0);
        const int c4 = (int)(lane & 15u) * 4;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's reads of the previous pass are done
#pragma unroll
            for (int bb = 0; bb < 2; ++bb)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    u32x4 q;
                    q.x = f2u(scale * acc[2 * h + bb][4 * g + 0]); q.y = f2u(scale * acc[2 * h + bb][4 * g + 1]);
                    q.z = f2u(scale * acc[2 * h + bb][4 * g + 2]); q.w = f2u(scale * acc[2 * h + bb][4 * g + 3]);
                    *(u32x4 *)(stg + (int)l32 * ST_STRIDE_F + bb * 32 + 8 * g + 4 * (int)half) = q;
                }
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's writes have landed before any lane reads
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int r = p * 4 + (int)(lane >> 4);
                const int32_t gr = row0 + r, gc = wcol0 + h * 64 + c4;
                if (gr < rows && gc < cols) {
                    const u32x4 q = *(const u32x4 *)(stg + r * ST_STRIDE_F + c4);
                    if (o_vec_ok) {
                        __builtin_nontemporal_store(q, (RANDES_GLOBAL u32x4 *)(out + (int64_t)gr * cols + gc));
                    } else {
                        const uint32_t w[4] = { q.x, q.y, q.z, q.w };
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (gc + j < cols) out[(int64_t)gr * cols + gc + j] = u2f(w[j]);
                    }
                }
            }
        }
    } else {
        // each wave stages and drains its own region: ordering inside one wave is all that is needed
        uint16_t *stg = (uint16_t *)sstage + wave * (LORA_TILE_M * ST_STRIDE);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wave's reads of the previous block are done
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                u32x2 q;
                q.x = pack_bf16x2(scale * acc[b][4 * g + 0], scale * acc[b][4 * g + 1]);
                q.y = pack_bf16x2(scale * acc[b][4 * g + 2], scale * acc[b][4 * g + 3]);
                *(u32x2 *)(stg + (int)l32 * ST_STRIDE + b * 32 + 8 * g + 4 * (int)half) = q;
            }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the wave's writes have landed before any lane reads
        RANDES_GLOBAL uint16_t *out = (RANDES_GLOBAL uint16_t *)it.out;
        const bool o_vec_ok = (cols % 8 == 0) && (((uintptr_t)it.out & 15u) == 0);
        const int c8 = (int)(lane & 15u) * 8;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int r = p * 4 + (int)(lane >> 4);
            const int32_t gr = row0 + r, gc = wcol0 + c8;
            if (gr < rows && gc < cols) {
                const u32x4 q = *(const u32x4 *)(stg + r * ST_STRIDE + c8);
                if (o_vec_ok) {
                    __builtin_nontemporal_store(q, (RANDES_GLOBAL u32x4 *)(out + (int64_t)gr * cols + gc));
                } else {
                    const uint32_t w[4] = { q.x, q.y, q.z, q.w };
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (gc + j < cols) out[(int64_t)gr * cols + gc + j] = (uint16_t)(w[j >> 1] >> (16 * (j & 1)));
                }
            }
        }
    }
  }   // row blocks
}

hipError_t launch_lora(const LoraItem *items_dev, int32_t n_items, const LoraSeg *segs_dev, const uint32_t *coarse_dev,
                       uint32_t n_tiles, int32_t max_seg, int32_t rank, float scale, int dt_ab, int dt_out, hipStream_t s)
{
    if (n_tiles == 0) return hipSuccess;
    const dim3 grid(n_tiles), block(WG);
    const int64_t slices = (int64_t)max_seg * ((rank + KCH - 1) / KCH);   // depth slices of the deepest matrix
    const int32_t row_tiles = lora_row_tiles(max_seg, rank);
#define RANDES_LORA(DA, DO, RES) hipLaunchKernelGGL((lora_kernel<DA, DO, RES>), grid, block, 0, s, items_dev, n_items, \
                                                    segs_dev, coarse_dev, rank, scale, row_tiles)
    if (dt_ab == DT_BF16) {
        // fragments of 1, up to 4 or up to 8 slices in registers (92 / ~150 / 245 registers per lane)
        const int res = slices <= 1 ? 1 : (slices <= 4 ? 4 : (slices <= LORA_RESIDENT_MAX ? LORA_RESIDENT_MAX : 0));
        if (dt_out == DT_BF16) {
            if (res == 1) RANDES_LORA(DT_BF16, DT_BF16, 1);
            else if (res == 4) RANDES_LORA(DT_BF16, DT_BF16, 4);
            else if (res == LORA_RESIDENT_MAX) RANDES_LORA(DT_BF16, DT_BF16, LORA_RESIDENT_MAX);
            else RANDES_LORA(DT_BF16, DT_BF16, 0);
        } else {
            if (res == 1) RANDES_LORA(DT_BF16, DT_F32, 1);
            else if (res == 4) RANDES_LORA(DT_BF16, DT_F32, 4);
            else if (res == LORA_RESIDENT_MAX) RANDES_LORA(DT_BF16, DT_F32, LORA_RESIDENT_MAX);
            else RANDES_LORA(DT_BF16, DT_F32, 0);
        }
    } else {
        if (dt_out == DT_BF16) {
            if (slices <= 1) RANDES_LORA(DT_F32, DT_BF16, 1); else RANDES_LORA(DT_F32, DT_BF16, 0);
        } else {
            if (slices <= 1) RANDES_LORA(DT_F32, DT_F32, 1); else RANDES_LORA(DT_F32, DT_F32, 0);
        }
    }
#undef RANDES_LORA
    return hipGetLastError();
}

}  // namespace randes
