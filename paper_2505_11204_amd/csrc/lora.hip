// LoRA deltas on the matrix cores (Sec. "Parameter Efficient Finetuning (PEFT) Model Compression":
// Theta_i = Theta_0 + lambda L_i with L_i = B_i A_i).
//
//   out = scale * sum over segments s of  B_s (rows x rank) * A_s (rank x cols) * D_s
//
// One segment without a sign flip is the plain materialisation L = scale * B A.  K segments, each
// with the sign diagonal D of its model, is the superposition of K adapters written once:
// sum_i (B_i A_i) D_i = [B_1 .. B_K] [A_1 D_1; ..; A_K D_K], a rank K*r contraction.
//
// Materialisation is bound by the output write, so the kernel is shaped after what the memory takes
// best, measured with plain fills: the chip should be writing few, compact regions at any moment.  A
// workgroup owns a band of 32 rows by NW * 64 columns (the whole row for the common widths) and walks
// down a few such bands; bands follow each other in memory order, and each of the 8 XCDs is given a
// contiguous eighth of them.  A wave owns 64 columns; the product is formed transposed (A^T as left
// operand, B^T as right) with 32x32 MFMAs, so a lane ends up with one output row and runs of adjacent
// columns, hands them to a row-major image of the band in LDS, and the workgroup then stores the image
// front to back, 16 bytes per lane.  Two images take turns, so filling one overlaps storing the other.
//
// Operands come straight from global memory into registers; nothing is staged and no barrier sits
// before the multiplies.  The right operand is 16 contiguous bytes of a row of B.  The left operand
// needs, per lane, the 8 depth values of one column of A, which lie a row apart in memory: a lane
// loads the dwords A[k][c], A[k][c+1] of a column pair for its 8 depth rows (neighbouring lanes read
// neighbouring dwords) and regroups them with byte permutes into the fragment of column c and the
// fragment of column c+1.  The two columns go to two different MFMA blocks: block E of a 64-column
// span holds its even columns, block O its odd ones, and that is exactly what makes a lane's results
// of the two blocks interleave into 8 adjacent output columns.  The sign flip is an XOR on the
// loaded dwords; the workgroup produces the sign bits of its band once, one lane per (model, 128
// columns), and keeps them in LDS.  Slices of 16 depth values are fetched a few slices ahead of the
// one being multiplied, through a ring of register buffers.  Deep products (high ranks) are bound by
// fetching and issuing rather than by the write: they run in small workgroups (four waves), of which
// several fit a CU, with two row blocks sharing every fetch of A.
//
// Superpositions of up to 8 depth slices (8 adapters of rank 16, 4 of rank 32, ...) go one step
// further: a wave's 64 columns do not change while its workgroup walks down the band, so the wave
// fetches, flips and regroups its fragments of A for all slices once and keeps them in registers
// (64 of them); a row block then costs 16 bytes per lane and slice of B, requested one block ahead,
// 16 MFMAs and the store.  Such a workgroup walks far (the launch is cut so that the chip is filled
// about once), which pays for the one fetch of A: 8 adapters on 72 matrices of 768 x 768 in 23 us
// against 45 us the streaming way.  Products of one or two slices take the same simple walk in the
// full-row bands (a few row blocks per workgroup): its waits are compiled exactly, where the ring's
// loop drains the wave's memory queue once per turn, which is worth 3-7 %.
//
// Operand layout of the 32x32 MFMAs: lane L supplies row (L % 32) of the left operand and column
// (L % 32) of the right operand for the depth slice owned by lane half (L / 32); accumulator
// register v of lane L is row 8*(v/4) + 4*(L/32) + (v%4), column L % 32 of the product.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_util.hpp"
#include "launch.hpp"
#include "philox.hpp"

namespace randes {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int KCH = LORA_DEPTH_SLICE;   // depth values per slice (one 32x32x16 MFMA, or eight 32x32x2)
constexpr int LORA_SIGN_SEGS = 32;      // segments whose sign bits a workgroup keeps in LDS
constexpr int LORA_RT2_SLICES = 4;     // depth slices from which two row blocks share every fetch of A
constexpr int LORA_RES_SLICES = 8;     // deepest product whose fragments of A stay in registers
constexpr double LORA_RES_FIXED = 5.0; // what such a workgroup spends before its first row block, in row blocks

struct LoraArgs {
    const LoraItem *items;
    const LoraSeg *segs;
    const uint32_t *wg_item;   // matrix of every workgroup tile
    uint32_t n_tiles;
    int32_t rank;
    int32_t rb;                // row-block groups one workgroup walks down
    float scale;
};

// What a wave fetches for one depth slice.
template <int DTAB, int NSPAN, int RT> struct SliceRaw;
template <int NSPAN, int RT> struct SliceRaw<DT_BF16, NSPAN, RT> {
    uint32_t a[NSPAN][8];   // per 64-column span: dwords (A[k][c], A[k][c+1]) of this lane's column pair, k = 8*half .. +7
    u32x4 b[RT];            // per row block: B[row][k0 + 8*half .. +7]
};
template <int NSPAN, int RT> struct SliceRaw<DT_F32, NSPAN, RT> {
    f32x2 a[NSPAN][8];      // per span and MFMA step st: (A[k][c], A[k][c+1]) at k = k0 + 2*st + half
    float b[RT][8];         // per row block and step: B[row][k0 + 2*st + half]
};

// Where a lane works.
struct LoraLane {
    int32_t rows, cols, rank;
    int32_t row0;          // first row of the workgroup's band
    int32_t wcol0;         // first column of this wave
    uint32_t half, l32;
};

// FAST addressing: a uniform base (segment pointer plus the slice's depth offset, in scalar registers)
// plus a 32-bit byte offset per lane and load that does not depend on the slice, so a wave keeps its
// offsets in registers for the whole kernel and a fetch is one base per operand plus the loads (the
// host sends matrices of 1 GiB and more down the other path).  Indices beyond the matrix are clamped
// to valid ones: what such lanes compute belongs to rows or columns that are never stored.  Only depth
// values beyond the rank must count as zero.  With the rank a multiple of 8 that can only be the
// upper 8 depth values of a segment's last slice: such a slice (`tail`) re-reads the lower 8 in their
// place and the multiply zeroes its B operand there.
template <int NSPAN, int RT> struct LoraOffsets {
    uint32_t a[NSPAN][8];   // bf16: ((8*half + j)*cols + c) * 2;  binary32: ((2*j + half)*cols + c) * 4
    uint32_t a_col[NSPAN];  // c * (2 or 4): the column part alone (tail slices)
    uint32_t b[RT];         // bf16: (row*rank + 8*half) * 2;  binary32: (row*rank + half) * 4
    uint32_t b_row[RT];     // row*rank * (2 or 4)
};

template <int DTAB, int NSPAN, int RT>
__device__ __forceinline__ void lora_column_offsets(const LoraLane &w, LoraOffsets<NSPAN, RT> &o)
{
    constexpr uint32_t EB = DTAB == DT_BF16 ? 2u : 4u;
#pragma unroll
    for (int sp = 0; sp < NSPAN; ++sp) {
        const int32_t c = w.wcol0 + sp * 64 + 2 * (int32_t)w.l32;
        const uint32_t cc = (uint32_t)(c < w.cols ? c : w.cols - 2);
        o.a_col[sp] = cc * EB;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t k = DTAB == DT_BF16 ? 8u * w.half + (uint32_t)j : 2u * (uint32_t)j + w.half;
            o.a[sp][j] = (k * (uint32_t)w.cols + cc) * EB;
        }
    }
}

template <int DTAB, int NSPAN, int RT>
__device__ __forceinline__ void lora_row_offsets(const LoraLane &w, LoraOffsets<NSPAN, RT> &o)
{
    constexpr uint32_t EB = DTAB == DT_BF16 ? 2u : 4u, KH = DTAB == DT_BF16 ? 8u : 1u;
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int32_t row = w.row0 + rt * 32 + (int32_t)w.l32;
        const uint32_t rc = (uint32_t)(row < w.rows ? row : w.rows - 1);
        o.b_row[rt] = rc * (uint32_t)w.rank * EB;
        o.b[rt] = o.b_row[rt] + KH * w.half * EB;
    }
}

// A pointer every lane agrees on, pinned to scalar registers (so that the per-lane part of an address
// stays a 32-bit offset beside it instead of being folded into 64-bit vector arithmetic).
__device__ __forceinline__ gcptr scalar_ptr(gcptr p)
{
    const uint64_t v = (uint64_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (gcptr)(((uint64_t)hi << 32) | (uint64_t)lo);
}

// Issue the loads of one depth slice (k0 .. k0 + 15 of segment S).  FAST fetches carry no arithmetic
// on what they load, and the same number of loads on every path, so that all loads of a slice (and
// of the slices fetched ahead) are in flight together and the wave waits for exactly the ones it needs.
template <int DTAB, int NSPAN, int RT, bool FAST>
__device__ __forceinline__ void lora_fetch(const LoraSeg &S, int32_t k0, const LoraLane &w, const LoraOffsets<NSPAN, RT> &off,
                                           SliceRaw<DTAB, NSPAN, RT> &raw)
{
    if constexpr (DTAB == DT_BF16) {
        if constexpr (FAST) {
            const gcptr abase = scalar_ptr((gcptr)S.A + (size_t)((uint32_t)k0 * (uint32_t)w.cols * 2u));
            const gcptr bbase = scalar_ptr((gcptr)S.B + (size_t)((uint32_t)k0 * 2u));
            if (k0 + 8 < w.rank) {   // uniform
#pragma unroll
                for (int sp = 0; sp < NSPAN; ++sp)
#pragma unroll
                    for (int j = 0; j < 8; ++j) raw.a[sp][j] = *(const RANDES_GLOBAL uint32_t *)(abase + off.a[sp][j]);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) raw.b[rt] = *(const RANDES_GLOBAL u32x4 *)(bbase + off.b[rt]);
            } else {                 // tail: both lane halves read depth rows k0 .. k0 + 7
                const uint32_t rowb = (uint32_t)w.cols * 2u;
#pragma unroll
                for (int sp = 0; sp < NSPAN; ++sp)
#pragma unroll
                    for (int j = 0; j < 8; ++j) raw.a[sp][j] = *(const RANDES_GLOBAL uint32_t *)(abase + (off.a_col[sp] + (uint32_t)j * rowb));
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) raw.b[rt] = *(const RANDES_GLOBAL u32x4 *)(bbase + off.b_row[rt]);
            }
        } else {
            const RANDES_GLOBAL uint16_t *Ap = (const RANDES_GLOBAL uint16_t *)S.A;
            const RANDES_GLOBAL uint16_t *Bp = (const RANDES_GLOBAL uint16_t *)S.B;
            const int32_t kb = k0 + 8 * (int32_t)w.half;
#pragma unroll
            for (int sp = 0; sp < NSPAN; ++sp) {
                const int32_t c = w.wcol0 + sp * 64 + 2 * (int32_t)w.l32;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int32_t k = kb + j;
                    uint32_t v = 0u;
                    if (k < w.rank) {
                        if (c < w.cols) v = Ap[(int64_t)k * w.cols + c];
                        if (c + 1 < w.cols) v |= (uint32_t)Ap[(int64_t)k * w.cols + c + 1] << 16;
                    }
                    raw.a[sp][j] = v;
                }
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int32_t row = w.row0 + rt * 32 + (int32_t)w.l32;
                uint32_t t[4] = {0u, 0u, 0u, 0u};
                if (row < w.rows) {
#pragma unroll
                    for (int j = 0; j < 8; ++j)
                        if (kb + j < w.rank) t[j >> 1] |= (uint32_t)Bp[(int64_t)row * w.rank + kb + j] << (16 * (j & 1));
                }
                raw.b[rt].x = t[0]; raw.b[rt].y = t[1]; raw.b[rt].z = t[2]; raw.b[rt].w = t[3];
            }
        }
    } else {
        if constexpr (FAST) {
            const gcptr abase = scalar_ptr((gcptr)S.A + (size_t)((uint32_t)k0 * (uint32_t)w.cols * 4u));
            const gcptr bbase = scalar_ptr((gcptr)S.B + (size_t)((uint32_t)k0 * 4u));
            if (k0 + 8 < w.rank) {   // uniform: all 16 depth rows exist
#pragma unroll
                for (int st = 0; st < 8; ++st) {
#pragma unroll
                    for (int sp = 0; sp < NSPAN; ++sp) raw.a[sp][st] = *(const RANDES_GLOBAL f32x2 *)(abase + off.a[sp][st]);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) raw.b[rt][st] = *(const RANDES_GLOBAL float *)(bbase + (off.b[rt] + (uint32_t)st * 8u));
                }
            } else {                 // tail: steps 4..7 re-read the depth rows of steps 0..3
#pragma unroll
                for (int st = 0; st < 8; ++st) {
#pragma unroll
                    for (int sp = 0; sp < NSPAN; ++sp) raw.a[sp][st] = *(const RANDES_GLOBAL f32x2 *)(abase + off.a[sp][st & 3]);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) raw.b[rt][st] = *(const RANDES_GLOBAL float *)(bbase + (off.b[rt] + (uint32_t)(st & 3) * 8u));
                }
            }
        } else {
            const RANDES_GLOBAL float *Ap = (const RANDES_GLOBAL float *)S.A;
            const RANDES_GLOBAL float *Bp = (const RANDES_GLOBAL float *)S.B;
#pragma unroll
            for (int sp = 0; sp < NSPAN; ++sp) {
                const int32_t c = w.wcol0 + sp * 64 + 2 * (int32_t)w.l32;
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const int32_t k = k0 + 2 * st + (int32_t)w.half;
                    f32x2 v = {0.0f, 0.0f};
                    if (k < w.rank) {
                        if (c < w.cols) v.x = Ap[(int64_t)k * w.cols + c];
                        if (c + 1 < w.cols) v.y = Ap[(int64_t)k * w.cols + c + 1];
                    }
                    raw.a[sp][st] = v;
                }
            }
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const int32_t row = w.row0 + rt * 32 + (int32_t)w.l32;
#pragma unroll
                for (int st = 0; st < 8; ++st) {
                    const int32_t k = k0 + 2 * st + (int32_t)w.half;
                    raw.b[rt][st] = (row < w.rows && k < w.rank) ? Bp[(int64_t)row * w.rank + k] : 0.0f;
                }
            }
        }
    }
}

// Sign bits of this lane's column pair in every span, one call of the generator per wave and segment:
// a wave's columns lie inside one 128-column generator block (NSPAN * 64 <= 128, aligned), and every
// operand of the call is wave-uniform.  Bit 0: column c, bit 1: column c + 1.
template <int NSPAN>
__device__ __forceinline__ void lora_pair_signs(const LoraSeg &S, const LoraLane &w, uint32_t (&bits)[NSPAN])
{
    if (!S.flip) {
#pragma unroll
        for (int sp = 0; sp < NSPAN; ++sp) bits[sp] = 0u;
        return;
    }
    const u32x4_t o = sign_block(S.key_lo, S.key_hi, S.layer_id, (uint32_t)w.wcol0 >> 7);
#pragma unroll
    for (int sp = 0; sp < NSPAN; ++sp) {
        const uint32_t rel = ((uint32_t)w.wcol0 & 127u) + (uint32_t)sp * 64u + 2u * w.l32;   // column inside the block
        const uint32_t sel = rel >> 5;
        const uint32_t word = sel == 0 ? o.w[0] : sel == 1 ? o.w[1] : sel == 2 ? o.w[2] : o.w[3];
        bits[sp] = (word >> (rel & 31u)) & 3u;
    }
}

// acc += (A D)^T-slice x B^T-slice for the slice fetched into `raw` (depth k0 .. k0 + 15 of its segment).
// FAST fetches bring operands of valid rows in place of depth rows beyond the rank: those are zeroed
// here, on the B side (element-wise fetches come zero-filled).
template <int DTAB, int NSPAN, int RT, bool FAST>
__device__ __forceinline__ void lora_multiply(const SliceRaw<DTAB, NSPAN, RT> &raw, const uint32_t (&bits)[NSPAN],
                                              int32_t k0, const LoraLane &w, f32x16 (&acc)[RT][2 * NSPAN])
{
    if constexpr (DTAB == DT_BF16) {
        u32x4 bq[RT];
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            bq[rt] = raw.b[rt];
            if constexpr (FAST) {
                const uint32_t ok = (k0 + 8 < w.rank || w.half == 0u) ? 0xffffffffu : 0u;
                bq[rt].x &= ok; bq[rt].y &= ok; bq[rt].z &= ok; bq[rt].w &= ok;
            }
        }
#pragma unroll
        for (int sp = 0; sp < NSPAN; ++sp) {
            const uint32_t m = ((bits[sp] & 1u) << 15) | ((bits[sp] & 2u) << 30);   // flips both halves of a pair dword
            u32x4 fe, fo;   // fragments of the even and the odd column: depth pairs (k, k+1) per dword
            uint32_t e[4], o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t d0 = raw.a[sp][2 * j] ^ m, d1 = raw.a[sp][2 * j + 1] ^ m;
                e[j] = __builtin_amdgcn_perm(d1, d0, 0x05040100u);   // low halves:  (A[k][c],   A[k+1][c])
                o[j] = __builtin_amdgcn_perm(d1, d0, 0x07060302u);   // high halves: (A[k][c+1], A[k+1][c+1])
            }
            fe.x = e[0]; fe.y = e[1]; fe.z = e[2]; fe.w = e[3];
            fo.x = o[0]; fo.y = o[1]; fo.z = o[2]; fo.w = o[3];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) {
                const bf16x8 bv = __builtin_bit_cast(bf16x8, bq[rt]);
                acc[rt][2 * sp] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fe), bv, acc[rt][2 * sp], 0, 0, 0);
                acc[rt][2 * sp + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fo), bv, acc[rt][2 * sp + 1], 0, 0, 0);
            }
        }
    } else {
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            const bool ok = !FAST || st < 4 || k0 + 8 < w.rank;   // uniform: steps 4..7 of a tail slice lie beyond the rank
#pragma unroll
            for (int sp = 0; sp < NSPAN; ++sp) {
                const uint32_t me = (bits[sp] & 1u) << 31, mo = (bits[sp] & 2u) << 30;
                const float ae = u2f(f2u(raw.a[sp][st].x) ^ me), ao = u2f(f2u(raw.a[sp][st].y) ^ mo);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    const float b = ok ? raw.b[rt][st] : 0.0f;
                    acc[rt][2 * sp] = __builtin_amdgcn_mfma_f32_32x32x2f32(ae, b, acc[rt][2 * sp], 0, 0, 0);
                    acc[rt][2 * sp + 1] = __builtin_amdgcn_mfma_f32_32x32x2f32(ao, b, acc[rt][2 * sp + 1], 0, 0, 0);
                }
            }
        }
    }
}

// Row pitch of the band's image in LDS: a few bytes more than the row, so that the lanes of a wave,
// which write 16 or 32 bytes each into 32 different rows, spread over the banks.
template <int DTO, int TN> struct StagePitch {
    static constexpr int value = (DTO == DT_BF16) ? TN * 2 + 32 : TN * 4 + 64;
};
template <int DTO, int TN> struct StageBytes {
    // bf16: 32 rows at once.  binary32: 16 rows at a time, in two passes.
    static constexpr int value = (DTO == DT_BF16 ? 32 : 16) * StagePitch<DTO, TN>::value;
};

// NW waves side by side, NB (even) blocks of 32 columns per wave.  A workgroup walks down P.rb
// consecutive groups of RT blocks of 32 rows inside its column band; the RT blocks of a group are
// multiplied together (they share every fetch of A), the groups one after the other.
// PF steps (a step = one depth slice of one group) are fetched ahead of the one being multiplied.
// FAST: every matrix of the launch has cols a multiple of 8, rank a multiple of 8 and operands
// aligned for the wide accesses (checked on the host); otherwise operands and results move by element.
// RES > 0: products of at most RES depth slices (superposed adapters, ranks of 64 to 128) keep the
// flipped, regrouped fragments of A of all their slices in registers: a wave's columns do not change
// while the workgroup walks down its band, so A is fetched once per workgroup instead of once per row
// group, and a row block costs the 16 bytes per lane and slice of B, the multiplies and the store.
template <int DTAB, int DTO, int NW, int NB, int RT, int PF, bool FAST, int RES = 0>
__global__ void __launch_bounds__(NW * 64) lora_kernel(const LoraArgs P)
{
    static_assert(NB % 2 == 0 && NB * 32 <= 128, "a wave's columns are whole 64-column spans inside one generator block");
    static_assert(RES == 0 || (DTAB == DT_BF16 && FAST && RT == 1 && NB == 2), "resident fragments: bf16 factors, wide accesses, one row block, one span");
    constexpr int NT = NW * 64, TN = NW * NB * 32, NSPAN = NB / 2;
    constexpr int PITCH = StagePitch<DTO, TN>::value;
    // two images take turns: a wave may fill the next one while others still store the previous one,
    // so one barrier per image (between filling and storing) is all the workgroup needs
    // (measured: the 512-column bands of 8 waves run faster with one image, all other shapes with two)
    constexpr int NIMG = NW == 8 ? 1 : 2;
    __shared__ __attribute__((aligned(16))) char stage2[NIMG][StageBytes<DTO, TN>::value];
    uint32_t image = 0;   // images filled so far (uniform)
    constexpr int NBLK = (TN + 127) / 128;   // generator blocks of 128 columns a band touches
    __shared__ uint32_t ssign[LORA_SIGN_SEGS * NBLK * 4];

    // XCD x (workgroups x, x + 8, ...) takes the x-th contiguous eighth of the tile sequence
    const uint32_t per_xcd = gridDim.x / 8u;
    const uint32_t bid = (blockIdx.x % 8u) * per_xcd + blockIdx.x / 8u;
    if (bid >= P.n_tiles) return;   // whole workgroup, before any barrier
    const LoraItem it = P.items[P.wg_item[bid]];
    const uint32_t idx = bid - it.tile_begin;
    const uint32_t tx = idx % it.tiles_x, ty = idx / it.tiles_x;
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lane = tid & 63u;
    LoraLane w;
    w.rows = it.rows; w.cols = it.cols; w.rank = P.rank;
    w.row0 = 0;
    const int32_t col0 = (int32_t)tx * TN;
    w.wcol0 = col0 + (int32_t)wave * NB * 32;
    w.half = lane >> 5; w.l32 = lane & 31u;
    const int32_t wband = (int32_t)wave * NB * 32;   // first column of the wave inside the band
    const float scale = P.scale;

    f32x16 acc[RT][NB];
    auto clear = [&]() {
#pragma unroll
        for (int rt = 0; rt < RT; ++rt)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[rt][b][v] = 0.0f;
    };
    clear();

    // ---- store one group of row blocks: band image in LDS, then front-to-back stores ----
    // A lane holds output row l32 of each row block and, in the accumulator pair (E, O) of span sp,
    // the columns wave*NB*32 + sp*64 + 16*g + 8*half + (0..7) of the band for g = 0..3: register
    // 4*g + i of E is column +2*i, of O column +2*i + 1.
    // The registers a store takes its address and data from are not free for anything else until the
    // store has completed.  Where stores and the next fetch alternate closely (RES), the pieces on
    // their way out keep registers of their own, which are written again only when the next row
    // block's pieces are ready, a whole row block later.
    constexpr int NPIN = RES > 0 ? 2 * NB : 1;
    u32x4 outq[1][NPIN];
    uint32_t outo[1][NPIN];
    if constexpr (RES > 0) {
#pragma unroll
        for (int h = 0; h < 1; ++h)
#pragma unroll
            for (int j = 0; j < NPIN; ++j) { outq[h][j] = u32x4{0u, 0u, 0u, 0u}; outo[h][j] = 0u; }
    }
    auto store_group = [&](int32_t grow0, auto set_tag) {
        constexpr int SET = decltype(set_tag)::value;
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
            const int32_t brow0 = grow0 + rt * 32;
            if ((RES == 0 || rt > 0) && brow0 >= w.rows) break;   // uniform (a group's first block always exists)
            if constexpr (DTO == DT_BF16) {
                char *stage = stage2[image % NIMG];
                ++image;
                if (NIMG == 1) __syncthreads();   // the previous image has been stored
#pragma unroll
                for (int sp = 0; sp < NSPAN; ++sp)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x4 q;
                        q.x = pack_bf16x2(scale * acc[rt][2 * sp][4 * g + 0], scale * acc[rt][2 * sp + 1][4 * g + 0]);
                        q.y = pack_bf16x2(scale * acc[rt][2 * sp][4 * g + 1], scale * acc[rt][2 * sp + 1][4 * g + 1]);
                        q.z = pack_bf16x2(scale * acc[rt][2 * sp][4 * g + 2], scale * acc[rt][2 * sp + 1][4 * g + 2]);
                        q.w = pack_bf16x2(scale * acc[rt][2 * sp][4 * g + 3], scale * acc[rt][2 * sp + 1][4 * g + 3]);
                        const int c = wband + sp * 64 + 16 * g + 8 * (int)w.half;
                        *(u32x4 *)(stage + (int)w.l32 * PITCH + c * 2) = q;
                    }
                __syncthreads();
                RANDES_GLOBAL uint16_t *out = (RANDES_GLOBAL uint16_t *)it.out;
                constexpr int CPR = TN / 8;   // 16-byte pieces per band row
#pragma unroll
                for (int j = 0; j < 32 * CPR / NT; ++j) {
                    const int piece = j * NT + (int)tid;
                    const int r = piece / CPR, c8 = (piece % CPR) * 8;
                    const int32_t gr = brow0 + r, gc = col0 + c8;
                    if constexpr (RES > 0) asm volatile("" : "+v"(outq[SET][j]), "+v"(outo[SET][j]));   // this set's last pieces lived until here
                    const bool inside = gr < w.rows && gc < w.cols;
                    if constexpr (RES > 0) {
                        // Every lane stores, whatever its piece: a store under a condition cannot be counted
                        // when the code is compiled, and every later wait for a fetched operand would then
                        // wait for the stores as well.  A lane whose piece lies outside the matrix stores the
                        // band's first piece, which always lies inside, once more: the same bytes to the same place.
                        const int rr = inside ? r : 0, cc = inside ? c8 : 0;
                        outq[SET][j] = *(const u32x4 *)(stage + rr * PITCH + cc * 2);
                        outo[SET][j] = ((uint32_t)(brow0 + rr) * (uint32_t)w.cols + (uint32_t)(col0 + cc)) * 2u;
                        asm volatile("" : "+v"(outq[SET][j]), "+v"(outo[SET][j]));
                        __builtin_nontemporal_store(outq[SET][j], (RANDES_GLOBAL u32x4 *)((gptr)it.out + outo[SET][j]));
                    } else if (inside) {
                        const u32x4 q = *(const u32x4 *)(stage + r * PITCH + c8 * 2);
                        if constexpr (FAST) {   // cols a multiple of 8 and out 16-byte aligned
                            __builtin_nontemporal_store(q, (RANDES_GLOBAL u32x4 *)((gptr)it.out + ((uint32_t)gr * (uint32_t)w.cols + (uint32_t)gc) * 2u));
                        } else {
                            const uint32_t t[4] = { q.x, q.y, q.z, q.w };
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (gc + e < w.cols) out[(int64_t)gr * w.cols + gc + e] = (uint16_t)(t[e >> 1] >> (16 * (e & 1)));
                        }
                    }
                }
            } else {
                RANDES_GLOBAL float *out = (RANDES_GLOBAL float *)it.out;
                constexpr int CPR = TN / 4;   // 16-byte pieces per band row
#pragma unroll
                for (int p = 0; p < 2; ++p) {   // rows 0..15 of the block, then rows 16..31
                    char *stage = stage2[image % NIMG];
                    ++image;
                    if (NIMG == 1) __syncthreads();
                    if ((int)(w.l32 >> 4) == p) {
#pragma unroll
                        for (int sp = 0; sp < NSPAN; ++sp)
#pragma unroll
                            for (int g = 0; g < 4; ++g) {
                                u32x4 q0, q1;
                                q0.x = f2u(scale * acc[rt][2 * sp][4 * g + 0]); q0.y = f2u(scale * acc[rt][2 * sp + 1][4 * g + 0]);
                                q0.z = f2u(scale * acc[rt][2 * sp][4 * g + 1]); q0.w = f2u(scale * acc[rt][2 * sp + 1][4 * g + 1]);
                                q1.x = f2u(scale * acc[rt][2 * sp][4 * g + 2]); q1.y = f2u(scale * acc[rt][2 * sp + 1][4 * g + 2]);
                                q1.z = f2u(scale * acc[rt][2 * sp][4 * g + 3]); q1.w = f2u(scale * acc[rt][2 * sp + 1][4 * g + 3]);
                                const int c = wband + sp * 64 + 16 * g + 8 * (int)w.half;
                                char *dst = stage + (int)(w.l32 & 15u) * PITCH + c * 4;
                                *(u32x4 *)dst = q0;
                                *(u32x4 *)(dst + 16) = q1;
                            }
                    }
                    __syncthreads();
#pragma unroll
                    for (int j = 0; j < 16 * CPR / NT; ++j) {
                        const int piece = j * NT + (int)tid;
                        const int r = piece / CPR, c4 = (piece % CPR) * 4;
                        const int32_t gr = brow0 + 16 * p + r, gc = col0 + c4;
                        if (gr < w.rows && gc < w.cols) {
                            const u32x4 q = *(const u32x4 *)(stage + r * PITCH + c4 * 4);
                            if constexpr (FAST) {   // cols a multiple of 4 and out 16-byte aligned
                                __builtin_nontemporal_store(q, (RANDES_GLOBAL u32x4 *)((gptr)it.out + ((uint32_t)gr * (uint32_t)w.cols + (uint32_t)gc) * 4u));
                            } else {
                                const uint32_t t[4] = { q.x, q.y, q.z, q.w };
#pragma unroll
                                for (int e = 0; e < 4; ++e)
                                    if (gc + e < w.cols) out[(int64_t)gr * w.cols + gc + e] = u2f(t[e]);
                            }
                        }
                    }
                }
            }
        }
    };

    // ---- the stream of (row group, segment, depth slice) steps of this workgroup ----
    const int32_t slices_per_seg = (P.rank + KCH - 1) / KCH;
    const int32_t n_seg = (int32_t)it.n_seg;
    const int32_t groups_total = (w.rows + 32 * RT - 1) / (32 * RT);
    const int32_t group0 = (int32_t)ty * P.rb;
    const int32_t n_groups = (groups_total - group0) < P.rb ? (groups_total - group0) : P.rb;
    const int32_t n_steps = n_groups * n_seg * slices_per_seg;
    // The tables are never written while the kernel runs: reading them through the constant address
    // space lets the look-ups stay scalar loads after the first results have been stored as well.
    typedef const __attribute__((address_space(4))) LoraSeg *ConstSegs;
    const ConstSegs segs = (ConstSegs)(uintptr_t)(P.segs + it.seg_begin);
    auto seg_at = [&](int32_t i) {
        LoraSeg S;
        S.B = segs[i].B; S.A = segs[i].A;
        S.key_lo = segs[i].key_lo; S.key_hi = segs[i].key_hi; S.layer_id = segs[i].layer_id; S.flip = segs[i].flip;
        return S;
    };
    // Sign bits of the band's columns for every segment, produced once per workgroup: one lane per
    // (segment, 128 columns), instead of one scalar evaluation of the generator per wave and slice (the
    // CU has a single scalar unit).  Products of more segments than the table holds use the scalar way.
    const bool signs_cached = n_seg <= LORA_SIGN_SEGS;
    if (signs_cached) {
        for (int32_t q = (int32_t)tid; q < n_seg * NBLK; q += NT) {
            const int32_t sgq = q / NBLK, blk = q % NBLK;
            const LoraSeg S = seg_at(sgq);
            u32x4_t o;
            o.w[0] = o.w[1] = o.w[2] = o.w[3] = 0u;
            if (S.flip) o = sign_block(S.key_lo, S.key_hi, S.layer_id, ((uint32_t)col0 >> 7) + (uint32_t)blk);
            ssign[q * 4 + 0] = o.w[0]; ssign[q * 4 + 1] = o.w[1]; ssign[q * 4 + 2] = o.w[2]; ssign[q * 4 + 3] = o.w[3];
        }
        __syncthreads();
    }
    struct Cursor { int32_t grp, sg, ks; };
    auto advance = [&](Cursor &c) {
        if (++c.ks == slices_per_seg) { c.ks = 0; if (++c.sg == n_seg) { c.sg = 0; ++c.grp; } }
    };
    // The cursor is the same in every lane; saying so keeps the segment look-ups and the generator on
    // the scalar unit (and out of the vector memory queue the operand fetches wait on).
    auto uni = [](int32_t v) { return (int32_t)__builtin_amdgcn_readfirstlane((uint32_t)v); };
    // Per-lane offsets change with the row group only; the fetch runs ahead of the multiply, so it
    // keeps offsets of its own.
    LoraOffsets<NSPAN, RT> off;
    int32_t off_grp = -1;
    if constexpr (FAST) lora_column_offsets<DTAB, NSPAN, RT>(w, off);
    if constexpr (RES > 0) {
        // The host sends here only launches whose every product has at most RES slices, rank a multiple
        // of 16 (no slice runs past its segment) and at most LORA_SIGN_SEGS segments.
        const int32_t n_sl = n_seg * slices_per_seg;
        auto slice_seg = [&](int s) {   // slices beyond the product repeat its last one and are not multiplied
            const int32_t sc = s < n_sl ? s : n_sl - 1;
            return sc / slices_per_seg;
        };
        auto slice_k0 = [&](int s) {
            const int32_t sc = s < n_sl ? s : n_sl - 1;
            return (sc % slices_per_seg) * KCH;
        };
        // Lane sl of every wave looks up the operand pointers of slice sl once; afterwards a slice's base
        // is two lane reads away (table look-ups inside the walk would put a chain of scalar loads and
        // waits in front of every row block).
        uint32_t a_lo, a_hi, b_lo, b_hi;
        {
            const int32_t my = (int32_t)(lane < (uint32_t)RES ? lane : 0u);
            const int32_t sg = slice_seg(my), k0 = slice_k0(my);
            const LoraSeg *gs = P.segs + it.seg_begin + sg;
            const uint64_t ap = (uint64_t)gs->A + (uint64_t)((uint32_t)k0 * (uint32_t)w.cols * 2u);
            const uint64_t bp = (uint64_t)gs->B + (uint64_t)((uint32_t)k0 * 2u);
            a_lo = (uint32_t)ap; a_hi = (uint32_t)(ap >> 32);
            b_lo = (uint32_t)bp; b_hi = (uint32_t)(bp >> 32);
        }
        auto lane_ptr = [](uint32_t lo, uint32_t hi, int sl) {
            // the lane read returns a signed word: through unsigned, or the low half's top bit would
            // smear over the high half
            const uint32_t l = (uint32_t)__builtin_amdgcn_readlane((int)lo, sl), h = (uint32_t)__builtin_amdgcn_readlane((int)hi, sl);
            return (gcptr)(((uint64_t)h << 32) | (uint64_t)l);
        };
        uint32_t araw[RES][8];
#pragma unroll
        for (int sl = 0; sl < RES; ++sl) {
            const gcptr abase = lane_ptr(a_lo, a_hi, sl);
#pragma unroll
            for (int j = 0; j < 8; ++j) araw[sl][j] = *(const RANDES_GLOBAL uint32_t *)(abase + off.a[0][j]);
        }
        // B of one row block: 16 bytes per lane and slice, rows clamped like everywhere on this path
        auto fetch_b = [&](int32_t grp, u32x4 (&dst)[RES]) {
            const int32_t g = grp < n_groups ? grp : n_groups - 1;
            const int32_t row = (group0 + g) * 32 + (int32_t)w.l32;
            const uint32_t rc = (uint32_t)(row < w.rows ? row : w.rows - 1);
            const uint32_t boff = (rc * (uint32_t)w.rank + 8u * w.half) * 2u;
#pragma unroll
            for (int sl = 0; sl < RES; ++sl) dst[sl] = *(const RANDES_GLOBAL u32x4 *)(lane_ptr(b_lo, b_hi, sl) + boff);
        };
        u32x4 bb[2][RES];
        fetch_b(0, bb[0]);
        // flip and regroup A once: fragments of the even and of the odd column of this lane's pair
        u32x4 fe[RES], fo[RES];
#pragma unroll
        for (int sl = 0; sl < RES; ++sl) {
            const int32_t sg = uni(slice_seg(sl));
            const uint32_t rel = (uint32_t)wband + 2u * w.l32;
            const uint32_t bits = (ssign[(sg * NBLK + (int32_t)(rel >> 7)) * 4 + (int32_t)((rel >> 5) & 3u)] >> (rel & 31u)) & 3u;
            const uint32_t m = ((bits & 1u) << 15) | ((bits & 2u) << 30);
            uint32_t e[4], o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t d0 = araw[sl][2 * j] ^ m, d1 = araw[sl][2 * j + 1] ^ m;
                e[j] = __builtin_amdgcn_perm(d1, d0, 0x05040100u);
                o[j] = __builtin_amdgcn_perm(d1, d0, 0x07060302u);
            }
            fe[sl].x = e[0]; fe[sl].y = e[1]; fe[sl].z = e[2]; fe[sl].w = e[3];
            fo[sl].x = o[0]; fo[sl].y = o[1]; fo[sl].z = o[2]; fo[sl].w = o[3];
        }
        auto block = [&](int32_t grp, const u32x4 (&b)[RES], auto set_tag) {
#pragma unroll
            for (int sl = 0; sl < RES; ++sl) {
                if (sl < n_sl) {   // uniform
                    const bf16x8 bv = __builtin_bit_cast(bf16x8, b[sl]);
                    acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fe[sl]), bv, acc[0][0], 0, 0, 0);
                    acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fo[sl]), bv, acc[0][1], 0, 0, 0);
                }
            }
            store_group((group0 + grp) * 32, set_tag);
            clear();
        };
        // The B of the next row block is requested before this one is multiplied and stored.  The first
        // block stands outside the loop, so that the loop is entered in the state every pass leaves
        // behind (one block's operands requested, the block before it on its way out): the waits inside
        // are compiled for what is really in flight, and no pass waits for the stores it follows.
        fetch_b(1, bb[1]);
        block(0, bb[0], std::integral_constant<int, 0>{});
        for (int32_t g = 1; g < n_groups; g += 2) {
            fetch_b(g + 1, bb[0]);
            block(g, bb[1], std::integral_constant<int, 0>{});
            if (g + 1 < n_groups) {   // uniform
                fetch_b(g + 2, bb[1]);
                block(g + 1, bb[0], std::integral_constant<int, 0>{});
            }
        }
        return;
    }
    auto fetch = [&](const Cursor &c, SliceRaw<DTAB, NSPAN, RT> &raw) {
        const int32_t grp = uni(c.grp);
        LoraLane wl = w;
        wl.row0 = (group0 + grp) * 32 * RT;
        if (FAST && grp != off_grp) { lora_row_offsets<DTAB, NSPAN, RT>(wl, off); off_grp = grp; }   // uniform
        const LoraSeg S = seg_at(uni(c.sg));
        lora_fetch<DTAB, NSPAN, RT, FAST>(S, uni(c.ks) * KCH, wl, off, raw);
    };
    auto consume = [&](const Cursor &c, const SliceRaw<DTAB, NSPAN, RT> &raw) {
        const int32_t sg = uni(c.sg), ks = uni(c.ks);
        LoraLane wl = w;
        wl.row0 = (group0 + uni(c.grp)) * 32 * RT;
        uint32_t bits[NSPAN];
        if (signs_cached) {
#pragma unroll
            for (int sp = 0; sp < NSPAN; ++sp) {
                const uint32_t rel = (uint32_t)wband + (uint32_t)sp * 64u + 2u * w.l32;   // this lane's column pair inside the band
                bits[sp] = (ssign[(sg * NBLK + (int32_t)(rel >> 7)) * 4 + (int32_t)((rel >> 5) & 3u)] >> (rel & 31u)) & 3u;
            }
        } else {
            const LoraSeg S = seg_at(sg);
            lora_pair_signs<NSPAN>(S, wl, bits);
        }
        lora_multiply<DTAB, NSPAN, RT, FAST>(raw, bits, ks * KCH, wl, acc);
        if (ks == slices_per_seg - 1 && sg == n_seg - 1) {   // the group is complete
            store_group(wl.row0, std::integral_constant<int, 0>{});
            clear();
        }
    };
    // A ring of PF + 1 buffers: step t multiplies buffer t mod (PF + 1) while the operands of steps
    // t + 1 .. t + PF are on their way, and no register of a buffer is touched between its fetch and
    // its multiply; while a group's results are stored, the next groups' operands are already in
    // flight.  Every step fetches, the last ones their own operands once more, so that the number of
    // loads in flight is the same on every path and a wave waits for exactly the oldest buffer's.
    constexpr int NBUF = PF + 1;
    SliceRaw<DTAB, NSPAN, RT> buf[NBUF];
    Cursor cur{0, 0, 0}, nxt{0, 0, 0};
    int32_t fetched = 0;   // steps whose fetch has been issued (the cursor stops at the last step)
    auto fetch_next = [&](SliceRaw<DTAB, NSPAN, RT> &raw) {
        if (fetched > 0 && fetched < n_steps) advance(nxt);
        fetch(nxt, raw);
        ++fetched;
    };
#pragma unroll
    for (int i = 0; i < PF; ++i) fetch_next(buf[i]);
    for (int32_t t = 0; t < n_steps; t += NBUF) {
#pragma unroll
        for (int i = 0; i < NBUF; ++i) {
            if (t + i < n_steps) {   // uniform
                fetch_next(buf[(i + PF) % NBUF]);
                consume(cur, buf[i]);
                advance(cur);
            }
        }
    }
}

// Band shapes a launch can take: nw waves of two column blocks each -> 768, 512 or 256 columns.
// Shallow products (materialisation: fewer than four depth slices) are bound by the output write and
// take the widest band that wastes no columns, whole rows where it can.  Deeper ones (superposed
// adapters, high ranks) spend their time fetching and multiplying and take small workgroups, of
// which more fit a CU, with two row blocks side by side, which halves the fetches of A.
LoraShape lora_choose_shape(const LoraItem *items, size_t n_items, int32_t max_seg, int32_t rank, bool f32_factors, bool fast)
{
    static const int cand[3] = { 12, 8, 4 };
    const int64_t slices = (int64_t)max_seg * ((rank + KCH - 1) / KCH);
    LoraShape best{};
    best.nb = 2;
    // Resident fragments: for superpositions of up to 8 slices (res = 8, 256-column bands, long walks),
    // and for products of one or two slices, which are bound by the write (res = 2: the band shape and
    // the short walks of the streaming kernel, 3-7 % faster than it).  A single adapter of rank 64, whose
    // one A stays in the caches anyway, measured 3-6 % faster the streaming way and keeps it.
    best.res = 0;
    if (fast && !f32_factors && rank % KCH == 0 && max_seg <= LORA_SIGN_SEGS) {
        if (slices <= 2) best.res = 2;
        else if (max_seg >= 2 && slices <= LORA_RES_SLICES) best.res = LORA_RES_SLICES;
    }
    best.rt = (slices >= LORA_RT2_SLICES && !f32_factors && !best.res) ? 2 : 1;
    const bool deep = slices >= 4 || best.res == LORA_RES_SLICES;
    double best_waste = -1.0;
    for (const int nw : cand) {
        if (deep && nw != 4) continue;
        const int64_t tn = (int64_t)nw * 64;
        double waste = 0.0;
        for (size_t q = 0; q < n_items; ++q) {
            const int64_t span = ((int64_t)items[q].cols + tn - 1) / tn * tn;
            waste += (double)(span - items[q].cols) * (double)items[q].rows;
        }
        if (best_waste < 0.0 || waste < best_waste) { best_waste = waste; best.nw = nw; }
    }
    best.tile_cols = best.nw * best.nb * 32;
    // A workgroup walks down rb groups of row blocks, so that the look-ups at its start and the first
    // fetch are paid once per rb stores; but the launch should still hand every CU a dozen workgroups.
    int64_t groups = 0;
    for (size_t q = 0; q < n_items; ++q)
        groups += (((int64_t)items[q].cols + best.tile_cols - 1) / best.tile_cols) *
                  (((int64_t)items[q].rows + 32 * best.rt - 1) / (32 * best.rt));
    const int64_t rb = groups / (256 * 12);
    best.rb = (int)(rb < 1 ? 1 : (rb > 8 ? 8 : rb));
    if (best.res == 2 && best.rb > 4) best.rb = 4;   // measured: walks of 3 or 4 row blocks
    if (best.res == LORA_RES_SLICES) {
        // Resident fragments pay the fetch of A once per workgroup: long walks, as long as the launch
        // still fills the chip's places for such workgroups about once.
        int best_rb = 1;
        double best_cost = -1.0;
        for (int cand_rb = 1; cand_rb <= 32; ++cand_rb) {
            int64_t wgs = 0;
            for (size_t q = 0; q < n_items; ++q)
                wgs += (((int64_t)items[q].cols + best.tile_cols - 1) / best.tile_cols) *
                       ((((int64_t)items[q].rows + 31) / 32 + cand_rb - 1) / cand_rb);
            const double rounds = (double)((wgs + 511) / 512);   // the chip holds 512 such workgroups at once, two per CU
            const double cost = rounds * (LORA_RES_FIXED + (double)cand_rb);   // in units of one row block
            if (best_cost < 0.0 || cost < best_cost) { best_cost = cost; best_rb = cand_rb; }
        }
        best.rb = best_rb;
    }
    return best;
}

// Steps fetched ahead of the multiply (binary32 operands fill the registers sooner).
constexpr int LORA_PF = 3, LORA_PF_F32 = 1;

template <int DTAB, int DTO, int NW, int RT>
static void lora_launch_one(const LoraArgs &a, bool fast, hipStream_t s)
{
    constexpr int PF = DTAB == DT_F32 ? LORA_PF_F32 : LORA_PF;
    const dim3 grid((a.n_tiles + 7u) / 8u * 8u), block(NW * 64);
    if (fast) hipLaunchKernelGGL((lora_kernel<DTAB, DTO, NW, 2, RT, PF, true>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((lora_kernel<DTAB, DTO, NW, 2, RT, PF, false>), grid, block, 0, s, a);
}

template <int DTAB, int DTO>
static hipError_t lora_dispatch(const LoraArgs &a, const LoraShape &sh, bool fast, hipStream_t s)
{
    if (sh.nb != 2) return hipErrorInvalidValue;
    if (sh.res) {
        if constexpr (DTAB == DT_BF16) {
            if (sh.rt != 1 || !fast) return hipErrorInvalidValue;
            const dim3 grid((a.n_tiles + 7u) / 8u * 8u), block(sh.nw * 64);
            if (sh.res == LORA_RES_SLICES && sh.nw == 4)
                hipLaunchKernelGGL((lora_kernel<DT_BF16, DTO, 4, 2, 1, LORA_PF, true, LORA_RES_SLICES>), grid, block, 0, s, a);
            else if (sh.res == 2 && sh.nw == 12)
                hipLaunchKernelGGL((lora_kernel<DT_BF16, DTO, 12, 2, 1, LORA_PF, true, 2>), grid, block, 0, s, a);
            else if (sh.res == 2 && sh.nw == 8)
                hipLaunchKernelGGL((lora_kernel<DT_BF16, DTO, 8, 2, 1, LORA_PF, true, 2>), grid, block, 0, s, a);
            else if (sh.res == 2 && sh.nw == 4)
                hipLaunchKernelGGL((lora_kernel<DT_BF16, DTO, 4, 2, 1, LORA_PF, true, 2>), grid, block, 0, s, a);
            else return hipErrorInvalidValue;
            return hipGetLastError();
        } else {
            return hipErrorInvalidValue;
        }
    }
    const int sel = sh.nw * 10 + sh.rt;
    switch (sel) {
    case 121: lora_launch_one<DTAB, DTO, 12, 1>(a, fast, s); break;
    case 81: lora_launch_one<DTAB, DTO, 8, 1>(a, fast, s); break;
    case 41: lora_launch_one<DTAB, DTO, 4, 1>(a, fast, s); break;
    case 42: if constexpr (DTAB == DT_BF16) { lora_launch_one<DTAB, DTO, 4, 2>(a, fast, s); break; } else return hipErrorInvalidValue;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_lora(const LoraItem *items_dev, const LoraSeg *segs_dev, const uint32_t *wg_item_dev,
                       uint32_t n_tiles, const LoraShape &shape, bool fast, int32_t rank, float scale,
                       int dt_ab, int dt_out, hipStream_t s)
{
    if (n_tiles == 0) return hipSuccess;
    LoraArgs a;
    a.items = items_dev; a.segs = segs_dev; a.wg_item = wg_item_dev;
    a.n_tiles = n_tiles; a.rank = rank; a.rb = shape.rb; a.scale = scale;
    if (dt_ab == DT_BF16) {
        if (dt_out == DT_BF16) return lora_dispatch<DT_BF16, DT_BF16>(a, shape, fast, s);
        return lora_dispatch<DT_BF16, DT_F32>(a, shape, fast, s);
    }
    if (dt_out == DT_BF16) return lora_dispatch<DT_F32, DT_BF16>(a, shape, fast, s);
    return lora_dispatch<DT_F32, DT_F32>(a, shape, fast, s);
}

}  // namespace randes
