// Small device-side helpers shared by the streaming and the LoRA kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace randes {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// Layer pointers reach the kernels through tables in memory, so the compiler cannot tell that
// they point to global memory and would fall back to flat addressing; say so explicitly.
#define RANDES_GLOBAL __attribute__((address_space(1)))
typedef const RANDES_GLOBAL char *gcptr;   // read-only global bytes
typedef RANDES_GLOBAL char *gptr;          // writable global bytes

constexpr int WG = 256;          // threads per workgroup
constexpr int WAVES = WG / 64;
constexpr int KREG_MAX = 8;      // merge: up to this many tasks keep their masks in registers
constexpr int MERGE_R = 4;       // merge: rows a wave loads before it stores (one burst)
constexpr int MERGE_WEIGHTS_R = 2;   // merge from weights: two streams per task, half the rows

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

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// Two binary32 values -> one dword of two bf16 (lo in bits 0..15) with gfx950's packed conversion
// (v_cvt_pk_bf16_f32): one instruction where the integer sequence above takes about fifteen for a
// pair.  Under the default rounding mode it returns bf16_rne(lo) | bf16_rne(hi) << 16 for every one
// of the 2^32 bit patterns in either half, NaNs, infinities and subnormals included (compared
// exhaustively on the device).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 v;
    v.x = lo; v.y = hi;
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

}  // namespace randes
