// Device-side helpers shared by the LCD kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lcd {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

// DPP controls: lane exchange inside a row of 16 lanes without touching LDS.
constexpr int kDppQuadXor1 = 0xB1;       // quad_perm:[1,0,3,2]
constexpr int kDppQuadXor2 = 0x4E;       // quad_perm:[2,3,0,1]
constexpr int kDppRowHalfMirror = 0x141; // lane j <-> 7-j inside each group of 8
constexpr int kDppRowMirror = 0x140;     // lane j <-> 15-j inside each row of 16

template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// (mask & a) | (~mask & b): one v_bfi_b32.
__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (mask & a) | (~mask & b); }

__device__ __forceinline__ half8 as_half8(uint4v v) { return __builtin_bit_cast(half8, v); }
__device__ __forceinline__ uint4v as_uint4(half8 v) { return __builtin_bit_cast(uint4v, v); }

// x / s in fp32 with IEEE division, rounded once more to fp16 (round to nearest even).
__device__ __forceinline__ _Float16 smooth_one(uint16_t xbits, float s)
{
    const float xf = (float)__builtin_bit_cast(_Float16, xbits);
    return (_Float16)__fdiv_rn(xf, s);
}

}  // namespace lcd
