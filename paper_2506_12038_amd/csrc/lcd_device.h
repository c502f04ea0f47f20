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

// Loads and stores of data that is touched once per kernel: the non-temporal hint keeps it from
// displacing what is reused.
template <class T> __device__ __forceinline__ T stream_load(const T *p) { return __builtin_nontemporal_load(p); }
template <class T> __device__ __forceinline__ void stream_store(T *p, T v) { __builtin_nontemporal_store(v, p); }

__device__ __forceinline__ half8 as_half8(uint4v v) { return __builtin_bit_cast(half8, v); }
__device__ __forceinline__ uint4v as_uint4(half8 v) { return __builtin_bit_cast(uint4v, v); }

// Smoothing of one activation: x * (1/s), the reciprocal in fp32 and accurate to 1 ulp (paper
// Sec. 4.1 folds the division into one multiplication by a stored reciprocal), the product
// rounded to fp16 by v_fma_mixlo_f16, which takes the fp16 operand as it is: one instruction
// instead of convert, multiply, convert.  Its last bit differs from that sequence on a few
// inputs, so EVERY smoothing in the library goes through this instruction: the fused and the
// ahead-of-time routes then agree bit for bit.  Exact when s is a power of two.
__device__ __forceinline__ _Float16 smooth_with(uint16_t xbits, float r)   // r = v_rcp_f32(s), shared by the caller
{
    const uint32_t a = xbits;
    uint32_t d;
    asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(a), "v"(r));
    return __builtin_bit_cast(_Float16, (uint16_t)d);
}
__device__ __forceinline__ _Float16 smooth_one(uint16_t xbits, float s) { return smooth_with(xbits, __builtin_amdgcn_rcpf(s)); }

// Two smoothed activations into one register in a single instruction each: v_fma_mix{lo,hi}_f16
// reads its first operand as the low or high fp16 half of a register, multiplies it by an fp32
// reciprocal and writes the fp32 product rounded to fp16 into the low / high half of the result --
// the arithmetic of smooth_one, two results per register.  LO_HALF / HI_HALF: which half of `a` / `b` holds the activation.
template <int LO_HALF, int HI_HALF>
__device__ __forceinline__ uint32_t smooth_pair(uint32_t a, float ra, uint32_t b, float rb)
{
    uint32_t d;
    if (LO_HALF == 0) asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(a), "v"(ra));
    else asm("v_fma_mixlo_f16 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(a), "v"(ra));
    if (HI_HALF == 0) asm("v_fma_mixhi_f16 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "+v"(d) : "v"(b), "v"(rb));
    else asm("v_fma_mixhi_f16 %0, %1, %2, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "+v"(d) : "v"(b), "v"(rb));
    return d;
}

// Input transformation of paper Sec. 4.1 (Eq. 10-11, b = 8), the smoothing and the quantisation
// fused: q = clip(round_half_even(x / (s * s_q)), -128, 127), every step in binary32 and the
// quotient correctly rounded (the rounding decision must be reproducible on the CPU, so a product
// with an approximate reciprocal is not enough).  The division is the usual reciprocal-refinement
// scheme, split so that the part which depends on the divisor alone is computed once per column
// and shared by all tokens: a Newton step on the hardware reciprocal, then per quotient a product
// and two residual corrections, all fused multiply-adds.  Valid without range scaling because
// |x| is a finite fp16 number and the caller keeps 2^-64 < s * s_q < 2^64.
struct Divisor {
    float neg_d;   // -(s * s_q)
    float y;       // refined reciprocal of s * s_q
};

__device__ __forceinline__ Divisor make_divisor(float s, float s_q)
{
    const float d = s * s_q;
    const float y0 = __builtin_amdgcn_rcpf(d);
    const float e = __builtin_fmaf(-d, y0, 1.0f);
    return Divisor{-d, __builtin_fmaf(e, y0, y0)};
}

// The code is returned as an fp16 number: integers up to 128 are exact.
__device__ __forceinline__ _Float16 quantise_one(uint16_t xbits, Divisor dv)
{
    const float xf = (float)__builtin_bit_cast(_Float16, xbits);
    float qt = xf * dv.y;
    qt = __builtin_fmaf(__builtin_fmaf(dv.neg_d, qt, xf), dv.y, qt);
    qt = __builtin_fmaf(__builtin_fmaf(dv.neg_d, qt, xf), dv.y, qt);
    float r = __builtin_rintf(qt);
    r = __builtin_fminf(__builtin_fmaxf(r, -128.0f), 127.0f);
    return (_Float16)r;
}

// a ^ (b & c): one v_bitop3_b32.
__device__ __forceinline__ uint32_t xor_and(uint32_t a, uint32_t b, uint32_t c) { return a ^ (b & c); }

}  // namespace lcd

namespace lcd {

// ---- register dequantiser: 16 packed indices -> two fp16 MFMA A operands ------------------
// v_perm_b32(hi4, lo4, sel): result byte b = byte sel[b] of the 8-byte pool {hi4 (4..7), lo4 (0..3)}.
__device__ __forceinline__ uint32_t perm(uint32_t hi4, uint32_t lo4, uint32_t sel) { return __builtin_amdgcn_perm(hi4, lo4, sel); }

// Per-row byte-split codebook: lo[0]/hi[0] hold the low/high bytes of centroids 0..3,
// lo[1]/hi[1] those of centroids 4..7 (3 bits only).
struct RowTables { uint32_t lo[2]; uint32_t hi[2]; };

// 3-bit only: the lane's two high-bit words, regrouped once per 64 weights so that the bits
// of selector t sit at one in-byte position of four bytes.
struct HighBits { uint32_t even, odd; };
__device__ __forceinline__ HighBits regroup_high(uint2v h)
{
    HighBits r;
    r.even = perm(h[1], h[0], 0x05040100u);
    r.odd = perm(h[1], h[0], 0x07060302u);
    return r;
}

// Decode low-plane word `p` (word d of the lane: 16 weights) into operand a=0 (weights
// 16d + [0,8)) and operand a=1 (weights 16d + [8,16)).  Register v of an operand holds the
// fp16 pair (weight v, weight 4+v) of its 8 weights, so the activation operand must use the
// slot order 0,4,1,5,2,6,3,7.
// One quarter of decode_word (selector T: weights T, 4+T of operand 0 and of operand 1), in its
// three dependent stages, so that a caller can interleave the stages of different quarters.
template <int BITS, int D, int T>
__device__ __forceinline__ uint32_t decode_select(uint32_t p, const HighBits &hb)
{
    uint32_t sel = (p >> (2 * T)) & 0x03030303u;
    if (BITS == 3) {
        constexpr int beta = 2 * D + (T >> 1);            // in-byte position of the high bit
        const uint32_t r = (T & 1) ? hb.odd : hb.even;
        const uint32_t sh = beta >= 2 ? (r >> (beta - 2)) : (r << (2 - beta));
        sel |= sh & 0x04040404u;
    }
    return sel;
}
template <int BITS>
__device__ __forceinline__ void decode_lookup(uint32_t sel, const RowTables &tb, uint32_t &lo, uint32_t &hi)
{
    lo = perm(BITS == 3 ? tb.lo[1] : 0u, tb.lo[0], sel);
    hi = perm(BITS == 3 ? tb.hi[1] : 0u, tb.hi[0], sel);
}
__device__ __forceinline__ void decode_interleave(uint32_t lo, uint32_t hi, uint32_t &o0, uint32_t &o1)
{
    o0 = perm(hi, lo, 0x05010400u);
    o1 = perm(hi, lo, 0x07030602u);
}
template <int BITS, int D, int T>
__device__ __forceinline__ void decode_quarter(uint32_t p, const HighBits &hb, const RowTables &tb, uint32_t &o0, uint32_t &o1)
{
    uint32_t lo, hi;
    decode_lookup<BITS>(decode_select<BITS, D, T>(p, hb), tb, lo, hi);
    decode_interleave(lo, hi, o0, o1);
}

// ---- 4 bits: 16 centroids per row ------------------------------------------------------------
// A byte permute reaches 8 table bytes, so the table is two pools (centroids 0..7 and 8..15):
// both are looked up with the low three index bits as selector and a third permute takes, byte by
// byte, the pool the fourth bit names.  p is the lane's low-plane word d, p2 its high-plane word d
// (same bit positions, index bits 2 and 3).
struct RowTables4 { uint32_t lo[4]; uint32_t hi[4]; };   // low / high bytes of centroids 4i..4i+3

template <int T>
__device__ __forceinline__ void decode_select4(uint32_t p, uint32_t p2, uint32_t &sel, uint32_t &pool)
{
    const uint32_t a = p >> (2 * T);
    const uint32_t b = T == 0 ? (p2 << 2) : (p2 >> (T == 0 ? 0 : 2 * T - 2));   // index bit 2 to in-byte bit 2
    const uint32_t c = T == 0 ? (p2 << 1) : (p2 >> (T == 0 ? 0 : 2 * T - 1));   // index bit 3 to in-byte bit 2
    sel = (a & 0x03030303u) | (b & 0x04040404u);
    pool = (c & 0x04040404u) | 0x03020100u;      // byte b: b (first pool) or 4 + b (second pool)
}
__device__ __forceinline__ void decode_lookup4(uint32_t sel, uint32_t pool, const RowTables4 &tb, uint32_t &lo, uint32_t &hi)
{
    lo = perm(perm(tb.lo[3], tb.lo[2], sel), perm(tb.lo[1], tb.lo[0], sel), pool);
    hi = perm(perm(tb.hi[3], tb.hi[2], sel), perm(tb.hi[1], tb.hi[0], sel), pool);
}
template <int T>
__device__ __forceinline__ void decode_quarter4(uint32_t p, uint32_t p2, const RowTables4 &tb, uint32_t &o0, uint32_t &o1)
{
    uint32_t sel, pool, lo, hi;
    decode_select4<T>(p, p2, sel, pool);
    decode_lookup4(sel, pool, tb, lo, hi);
    decode_interleave(lo, hi, o0, o1);
}
// Same operand convention as decode_word below.
__device__ __forceinline__ void decode_word4(uint32_t p, uint32_t p2, const RowTables4 &tb, uint4v &op0, uint4v &op1)
{
    uint32_t a, b;
    decode_quarter4<0>(p, p2, tb, a, b); op0[0] = a; op1[0] = b;
    decode_quarter4<1>(p, p2, tb, a, b); op0[1] = a; op1[1] = b;
    decode_quarter4<2>(p, p2, tb, a, b); op0[2] = a; op1[2] = b;
    decode_quarter4<3>(p, p2, tb, a, b); op0[3] = a; op1[3] = b;
}

template <int BITS, int D>
__device__ __forceinline__ void decode_word(uint32_t p, const HighBits &hb, const RowTables &tb, uint4v &op0, uint4v &op1)
{
    uint32_t a, b;
    decode_quarter<BITS, D, 0>(p, hb, tb, a, b); op0[0] = a; op1[0] = b;
    decode_quarter<BITS, D, 1>(p, hb, tb, a, b); op0[1] = a; op1[1] = b;
    decode_quarter<BITS, D, 2>(p, hb, tb, a, b); op0[2] = a; op1[2] = b;
    decode_quarter<BITS, D, 3>(p, hb, tb, a, b); op0[3] = a; op1[3] = b;
}

}  // namespace lcd
