// Decode path (M <= 16) of the smoothed table-lookup product, gfx950.
//
// Single-token kernel ("bucket" kernel).  The lookup + accumulation of paper Sec. 4.2 is done
// by the sparse matrix core: v_smfmac_f32_16x16x64_f16 multiplies, for each of 16 rows, 32
// values of its A operand with rows of a dense B operand *selected by 2-bit indices held in a
// register*.  Feeding
//     A     = the smoothed activations xs[k]          (the same for all 16 output rows),
//     index = the packed 2-bit weight indices, as stored in memory (no decode instruction),
//     B     = a constant 0/1 matrix that routes "index == c" to accumulator column c,
// makes accumulator column c of row n the centroid bucket sum  S[n][c] = sum_{k: idx[n][k]==c} xs[k];
// the output is y[n] = sum_c C[n][c] * S[n][c], four multiplies per row at the very end.
// For 3-bit indices the third bit h flips the sign of the activation in a second pass that
// lands in columns 4..7:  C[n][4h+l] = P[n][l] + (1-2h) Q[n][l]  gives
//     y[n] = sum_l P[n][l] * (sum_{k: l_k==l} xs[k]) + Q[n][l] * (sum_{k: l_k==l} (-1)^{h_k} xs[k]).
// The sign flip is one shift and one v_bfi_b32 per pair of weights.
//
// Work split: a wave owns CH consecutive 256-column chunks and keeps their activations in
// registers for its whole life; it walks over row tiles (16 rows), streaming CH KiB-sized
// contiguous pieces of the packed matrix per tile.  The waves of a workgroup cover a
// contiguous K range; their partial outputs meet in LDS (fixed order).  If K needs more than
// one workgroup, fp32 partials go to the workspace and a second kernel adds them.
#include <hip/hip_runtime.h>
#include "lcd_internal.h"
#include "lcd_device.h"

namespace lcd {


constexpr int kMaxWaves = 8;

// Buffer resources give branch-free predication: a lane whose offset is past the end of the
// buffer reads zeros and touches no memory.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}
constexpr uint32_t kOob = 0xFFFFFFF0u;

template <int BITS, int CH>
struct TileRegs {
    uint4v lo[CH];   // 2-bit plane: the lane's 64 low index pairs per chunk
    uint2v hi[CH];   // 3-bit only: the lane's 64 high bits per chunk
    float4v cf;      // per-bucket multipliers of this lane's 4 rows (lanes j < NC), else 0
};

// Issue the loads of row tile t (nothing is read if t >= nt or a chunk is not this wave's).
template <int BITS, int CH>
__device__ __forceinline__ void load_tile(TileRegs<BITS, CH> &r, __amdgpu_buffer_rsrc_t packed, __amdgpu_buffer_rsrc_t lutA,
                                          int t, int nt, uint32_t tile_stride, const uint32_t (&choff)[CH], int lane)
{
    constexpr int NC = BITS == 2 ? 4 : 8;
    const bool tv = t < nt;
    const uint32_t toff = (uint32_t)t * tile_stride;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        const bool v = tv && choff[ch] != kOob;
        const uint32_t o = toff + choff[ch];
        r.lo[ch] = __builtin_amdgcn_raw_buffer_load_b128(packed, v ? o + 16 * lane : kOob, 0, 0);
        if (BITS == 3) r.hi[ch] = __builtin_amdgcn_raw_buffer_load_b64(packed, v ? o + 1024 + 8 * lane : kOob, 0, 0);
    }
    const int j = lane & 15, bq = lane >> 4;
    const uint32_t lo = ((uint32_t)(4 * t + bq) * NC + j) * 16;
    r.cf = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(lutA, (tv && j < NC) ? lo : kOob, 0, 0));
}

template <int BITS, int CH>
__global__ void __launch_bounds__(kMaxWaves * 64, 1)
gemv_bucket_kernel(const uint8_t *__restrict__ packed_, const float *__restrict__ lutA_, const uint16_t *__restrict__ x,
                   const float *__restrict__ s, uint16_t *__restrict__ y, float *__restrict__ partial,
                   int N, int K, int chunks_per_split, int splits)
{
    constexpr int NC = BITS == 2 ? 4 : 8;
    constexpr uint32_t TB = BITS == 2 ? 1024 : 1536;
    __shared__ __attribute__((aligned(16))) _Float16 xs_lds[kMaxWaves * CH * 256];
    __shared__ __attribute__((aligned(16))) float part[2][kMaxWaves][16];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int q = lane >> 4, j = lane & 15, bq = lane >> 4;
    const int kc = K / kTileCols, nt = N / kTileRows;
    const int split = blockIdx.y;
    const int split_c0 = split * chunks_per_split;
    const int split_c1 = min(kc, split_c0 + chunks_per_split);
    const int c_begin = split_c0 + wave * CH;
    const __amdgpu_buffer_rsrc_t packed = make_rsrc(packed_, (uint32_t)nt * (uint32_t)kc * TB);
    const __amdgpu_buffer_rsrc_t lutA = make_rsrc(lutA_, (uint32_t)N * NC * 4);
    const uint32_t tile_stride = (uint32_t)kc * TB;
    uint32_t choff[CH];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) choff[ch] = (c_begin + ch < split_c1) ? (uint32_t)(c_begin + ch) * TB : kOob;

    // ---- prologue: smoothed activations of this workgroup's K range -> LDS -> registers.
    // Its loads go first (they head the longest dependency chain), then the first tiles'.
    const int stride = gridDim.x;
    int t = blockIdx.x;
    TileRegs<BITS, CH> r0, r1, r2;
    {
        const int k0 = split_c0 * kTileCols, groups = (split_c1 - split_c0) * (kTileCols / 8);
        for (int g = threadIdx.x; g < groups; g += blockDim.x) {
            const uint4v xv = *reinterpret_cast<const uint4v *>(x + k0 + 8 * g);
            const float4v s0 = *reinterpret_cast<const float4v *>(s + k0 + 8 * g);
            const float4v s1 = *reinterpret_cast<const float4v *>(s + k0 + 8 * g + 4);
            half8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e)
                o[e] = smooth_one((uint16_t)(xv[e >> 1] >> (16 * (e & 1))), e < 4 ? s0[e] : s1[e - 4]);
            *reinterpret_cast<half8 *>(&xs_lds[8 * g]) = o;
        }
    }
    load_tile<BITS, CH>(r0, packed, lutA, t, nt, tile_stride, choff, lane);
    load_tile<BITS, CH>(r1, packed, lutA, t + stride, nt, tile_stride, choff, lane);
    __syncthreads();
    uint4v A[CH][8];
    uint4v nA[BITS == 3 ? CH : 1][8];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch)
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            uint4v v = {0u, 0u, 0u, 0u};
            if (choff[ch] != kOob) v = *reinterpret_cast<const uint4v *>(&xs_lds[(wave * CH + ch) * 256 + 64 * q + 8 * g]);
            A[ch][g] = v;
            if (BITS == 3) nA[ch][g] = v ^ 0x80008000u;
        }
    // constant routing matrices: B1 sends index c to column c, B2 to column 4 + c
    half16 B1, B2;
#pragma unroll
    for (int b = 0; b < 16; ++b) {
        B1[b] = ((b & 3) == j) ? (_Float16)1.0f : (_Float16)0.0f;
        B2[b] = ((b & 3) + 4 == j) ? (_Float16)1.0f : (_Float16)0.0f;
    }

    auto process = [&](const TileRegs<BITS, CH> &r, int tile, int buf) {
        float4v acc[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[u] = float4v{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int idxreg = (int)r.lo[ch][d];
                // half a = 0 uses index bits [15:0], a = 1 bits [31:16]
                if (BITS == 2) {
                    acc[(2 * d) & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d]), B1, acc[(2 * d) & 3], idxreg, 0, 0);
                    acc[(2 * d + 1) & 3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d + 1]), B1, acc[(2 * d + 1) & 3], idxreg, 0, 1);
                } else {
                    acc[0] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d]), B1, acc[0], idxreg, 0, 0);
                    acc[1] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d + 1]), B1, acc[1], idxreg, 0, 1);
#pragma unroll
                    for (int a = 0; a < 2; ++a) {
                        const uint32_t hp = r.hi[ch][a];
                        uint4v f;
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            // pair v of this operand: high bits sit 16 apart; move them to bits 15 / 31
                            const int sh = 15 - (8 * (v >> 1) + 2 * d + (v & 1));
                            f[v] = bfi(hp << sh, nA[ch][2 * d + a][v], A[ch][2 * d + a][v]);
                        }
                        if (a == 0) acc[2] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f), B2, acc[2], idxreg, 0, 0);
                        else        acc[3] = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f), B2, acc[3], idxreg, 0, 1);
                    }
                }
            }
        }
        // bucket sums -> outputs: multiply by the codebook-derived factors, add the NC columns
        float4v p;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v = ((acc[0][u] + acc[1][u]) + (acc[2][u] + acc[3][u])) * r.cf[u];
            v += dpp_f32<kDppQuadXor1>(v);
            v += dpp_f32<kDppQuadXor2>(v);
            if (NC == 8) v += dpp_f32<kDppRowHalfMirror>(v);
            p[u] = v;
        }
        if (j == 0) *reinterpret_cast<float4v *>(&part[buf][wave][4 * bq]) = p;
        __syncthreads();
        if (threadIdx.x < 16) {
            float sum = 0.f;
            for (int w = 0; w < nwaves; ++w) sum += part[buf][w][threadIdx.x];
            const size_t o = (size_t)tile * kTileRows + threadIdx.x;
            if (splits == 1) y[o] = __builtin_bit_cast(uint16_t, (_Float16)sum);
            else partial[(size_t)split * N + o] = sum;
        }
    };

    // three register sets rotate: two tiles are always in flight behind the one being consumed
    while (true) {
        load_tile<BITS, CH>(r2, packed, lutA, t + 2 * stride, nt, tile_stride, choff, lane);
        process(r0, t, 0);
        t += stride;
        if (t >= nt) break;
        load_tile<BITS, CH>(r0, packed, lutA, t + 2 * stride, nt, tile_stride, choff, lane);
        process(r1, t, 1);
        t += stride;
        if (t >= nt) break;
        load_tile<BITS, CH>(r1, packed, lutA, t + 2 * stride, nt, tile_stride, choff, lane);
        process(r2, t, 0);
        t += stride;
        if (t >= nt) break;
        load_tile<BITS, CH>(r2, packed, lutA, t + 2 * stride, nt, tile_stride, choff, lane);
        process(r0, t, 1);
        t += stride;
        if (t >= nt) break;
        load_tile<BITS, CH>(r0, packed, lutA, t + 2 * stride, nt, tile_stride, choff, lane);
        process(r1, t, 0);
        t += stride;
        if (t >= nt) break;
        load_tile<BITS, CH>(r1, packed, lutA, t + 2 * stride, nt, tile_stride, choff, lane);
        process(r2, t, 1);
        t += stride;
        if (t >= nt) break;
    }
}

// ---- batched decode kernel (2 <= M <= 16) ---------------------------------------------------
// Same work split as the bucket kernel, but the 16 columns of the matrix core's output tile are
// the tokens: the packed indices are dequantised in registers (v_perm_b32 through per-row
// byte-split codebook tables) into the A operand of v_mfma_f32_16x16x32_f16, and the smoothed
// activations of the wave's K range stay in registers as B operands.
template <int BITS, int CH>
struct DenseTileRegs {
    uint4v lo[CH];
    uint2v hi[CH];
    RowTables tb;
};

template <int BITS, int CH>
__device__ __forceinline__ void load_dense_tile(DenseTileRegs<BITS, CH> &r, const uint8_t *__restrict__ packed,
                                                const uint8_t *__restrict__ lutB, int t, int kc, int c_begin, int nch, int lane)
{
    constexpr size_t TB = BITS == 2 ? 1024 : 1536;
    const uint8_t *base = packed + ((size_t)t * kc + c_begin) * TB;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        if (ch < nch) {
            r.lo[ch] = __builtin_nontemporal_load(reinterpret_cast<const uint4v *>(base + ch * TB + 16 * lane));
            if (BITS == 3) r.hi[ch] = __builtin_nontemporal_load(reinterpret_cast<const uint2v *>(base + ch * TB + 1024 + 8 * lane));
        }
    }
    const size_t row = (size_t)t * kTileRows + (lane & 15);
    if (BITS == 2) {
        const uint2v v = *reinterpret_cast<const uint2v *>(lutB + row * 8);
        r.tb.lo[0] = v[0]; r.tb.hi[0] = v[1]; r.tb.lo[1] = 0; r.tb.hi[1] = 0;
    } else {
        const uint4v v = *reinterpret_cast<const uint4v *>(lutB + row * 16);
        r.tb.lo[0] = v[0]; r.tb.lo[1] = v[1]; r.tb.hi[0] = v[2]; r.tb.hi[1] = v[3];
    }
}

template <int BITS, int CH, int D>
__device__ __forceinline__ void dense_word(const DenseTileRegs<BITS, CH> &r, int ch, const HighBits &hb,
                                           const uint4v (&Bx)[CH][8], float4v (&acc)[2])
{
    uint4v op0, op1;
    decode_word<BITS, D>(r.lo[ch][D], hb, r.tb, op0, op1);
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op0), as_half8(Bx[ch][2 * D]), acc[0], 0, 0, 0);
    acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op1), as_half8(Bx[ch][2 * D + 1]), acc[1], 0, 0, 0);
}

template <int BITS, int CH>
__global__ void __launch_bounds__(kMaxWaves * 64, 1)
gemv_dense_kernel(const uint8_t *__restrict__ packed, const uint8_t *__restrict__ lutB, const _Float16 *__restrict__ xs,
                  uint16_t *__restrict__ y, float *__restrict__ partial, int M, int N, int K, int chunks_per_split, int splits)
{
    __shared__ __attribute__((aligned(16))) float part[2][kMaxWaves][16][16];  // [buf][wave][token][row]

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int q = lane >> 4, j = lane & 15, bq = lane >> 4;
    const int kc = K / kTileCols, nt = N / kTileRows;
    const int split = blockIdx.y;
    const int split_c0 = split * chunks_per_split;
    const int split_c1 = min(kc, split_c0 + chunks_per_split);
    const int c_begin = split_c0 + wave * CH;
    const int nch = max(0, min(CH, split_c1 - c_begin));

    DenseTileRegs<BITS, CH> r0, r1;
    int t = blockIdx.x;
    if (t < nt) load_dense_tile<BITS, CH>(r0, packed, lutB, t, kc, c_begin, nch, lane);

    // B operands: lane (q, token j) keeps xs[j][chunk*256 + 64q + 8g + 0..7] for every chunk it owns
    uint4v Bx[CH][8];
#pragma unroll
    for (int ch = 0; ch < CH; ++ch)
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            uint4v v = {0u, 0u, 0u, 0u};
            if (ch < nch && j < M)
                v = *reinterpret_cast<const uint4v *>(xs + (size_t)j * K + (size_t)(c_begin + ch) * kTileCols + 64 * q + 8 * g);
            Bx[ch][g] = v;
        }

    auto process = [&](const DenseTileRegs<BITS, CH> &r, int tile, int buf) {
        float4v acc[2] = {float4v{0.f, 0.f, 0.f, 0.f}, float4v{0.f, 0.f, 0.f, 0.f}};
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            if (ch < nch) {
                HighBits hb{0u, 0u};
                if (BITS == 3) hb = regroup_high(r.hi[ch]);
                dense_word<BITS, CH, 0>(r, ch, hb, Bx, acc);
                dense_word<BITS, CH, 1>(r, ch, hb, Bx, acc);
                dense_word<BITS, CH, 2>(r, ch, hb, Bx, acc);
                dense_word<BITS, CH, 3>(r, ch, hb, Bx, acc);
            }
        }
        // accumulator: lane (bq, j) holds rows 4bq..4bq+3 of token j
        const float4v p = acc[0] + acc[1];
        *reinterpret_cast<float4v *>(&part[buf][wave][j][4 * bq]) = p;
        __syncthreads();
        {
            const int e = threadIdx.x;
            for (int o = e; o < 16 * M; o += blockDim.x) {
                const int m = o >> 4, row = o & 15;
                float sum = 0.f;
                for (int w = 0; w < nwaves; ++w) sum += part[buf][w][m][row];
                const size_t dst = (size_t)m * N + (size_t)tile * kTileRows + row;
                if (splits == 1) y[dst] = __builtin_bit_cast(uint16_t, (_Float16)sum);
                else partial[(size_t)split * M * N + dst] = sum;
            }
        }
    };

    const int stride = gridDim.x;
    while (t < nt) {
        const int t1 = t + stride;
        if (t1 < nt) load_dense_tile<BITS, CH>(r1, packed, lutB, t1, kc, c_begin, nch, lane);
        process(r0, t, 0);
        if (t1 >= nt) break;
        const int t2 = t1 + stride;
        if (t2 < nt) load_dense_tile<BITS, CH>(r0, packed, lutB, t2, kc, c_begin, nch, lane);
        process(r1, t1, 1);
        t = t2;
    }
}

template <int BITS, int CH>
static int launch_bucket(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                         float *partial, int N, int K, const GemvPlan &plan, hipStream_t stream)
{
    hipLaunchKernelGGL((gemv_bucket_kernel<BITS, CH>), dim3(plan.grid_x, plan.splits), dim3(plan.waves * 64), 0, stream,
                       (const uint8_t *)packed, (const float *)lut, x, s, y, partial, N, K, plan.chunks_per_split, plan.splits);
    return (int)hipGetLastError();
}

int launch_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, void *workspace, const GemvPlan &plan, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    float *partial = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + plan.xs_bytes);
    if (M == 1) {
        int e = bits == 2 ? launch_bucket<2, 4>(packed, lut, x, s, y, partial, N, K, plan, stream)
                          : launch_bucket<3, 2>(packed, lut, x, s, y, partial, N, K, plan, stream);
        if (e) return e;
        if (plan.splits > 1) return launch_reduce(partial, y, plan.splits, (long long)N, stream);
        return 0;
    }
    // batched: smooth once into the workspace (dequantiser slot order), then the dense kernel
    _Float16 *xs = reinterpret_cast<_Float16 *>(workspace);
    if (int e = launch_smooth(x, s, xs, M, M, K, 0, stream)) return e;
    const uint8_t *lutB = static_cast<const uint8_t *>(lut) + (size_t)N * (bits == 2 ? 4 : 8) * 4;
    const dim3 grid(plan.grid_x, plan.splits), block(plan.waves * 64);
    if (bits == 2)
        hipLaunchKernelGGL((gemv_dense_kernel<2, 4>), grid, block, 0, stream, (const uint8_t *)packed, lutB, xs, y, partial,
                           M, N, K, plan.chunks_per_split, plan.splits);
    else
        hipLaunchKernelGGL((gemv_dense_kernel<3, 4>), grid, block, 0, stream, (const uint8_t *)packed, lutB, xs, y, partial,
                           M, N, K, plan.chunks_per_split, plan.splits);
    if (int e = (int)hipGetLastError()) return e;
    if (plan.splits > 1) return launch_reduce(partial, y, plan.splits, (long long)M * N, stream);
    return 0;
}

}  // namespace lcd
