// Prefill path (M >= 64; any M >= 1 accepted) of the smoothed table-lookup product, gfx950.
//
// This path is a dense contraction, so it runs on v_mfma_f32_16x16x32_f16 with fp32
// accumulators.  Output tile per workgroup: 256 rows x 128 tokens; wave w owns rows
// [64w, 64w+64) (4 row tiles) and all 128 tokens (8 token tiles): 32 accumulators.
//   * A operand = weights.  Each lane dequantises its own packed indices in registers
//     (v_perm_b32 through the row's byte-split codebook), exactly the lane <-> (row, k) mapping
//     of the packed layout, so weights never pass through LDS.
//   * B operand = smoothed activations xs = x / s (fp16), prepared once per call by a small
//     kernel in MFMA-operand order, so that the slice one workgroup needs per 256-column chunk
//     is one contiguous 64 KiB block.  It is copied global -> LDS with direct-to-LDS loads,
//     double buffered, and every wave reads its B operands from LDS (16 bytes per lane,
//     conflict-free).
// Each decoded A operand is used for 8 token tiles, each B operand for 4 row tiles.
#include <hip/hip_runtime.h>
#include "lcd_internal.h"
#include "lcd_device.h"

namespace lcd {

constexpr int kGemmWaves = 4;
constexpr int kGemmRowTiles = 4;     // per wave
constexpr int kGemmTokTiles = 8;     // per workgroup (shared by its waves)
constexpr int kGemmTokens = 16 * kGemmTokTiles;
constexpr int kStageBytes = kGemmTokTiles * 8 * 1024;  // 64 KiB: 8 token tiles x 8 k-steps x 1 KiB

typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(1))) const uint32_t glb_u32;

template <int BITS>
struct GemmTileRegs {
    uint4v lo[kGemmRowTiles];
    uint2v hi[kGemmRowTiles];
};

template <int BITS>
__device__ __forceinline__ void load_gemm_tiles(GemmTileRegs<BITS> &r, const uint8_t *__restrict__ packed, int t0, int nt,
                                                int kc, int c, int lane)
{
    constexpr size_t TB = BITS == 2 ? 1024 : 1536;
#pragma unroll
    for (int rt = 0; rt < kGemmRowTiles; ++rt) {
        if (t0 + rt < nt) {
            const uint8_t *base = packed + ((size_t)(t0 + rt) * kc + c) * TB;
            r.lo[rt] = *reinterpret_cast<const uint4v *>(base + 16 * lane);
            if (BITS == 3) r.hi[rt] = *reinterpret_cast<const uint2v *>(base + 1024 + 8 * lane);
        } else {
            r.lo[rt] = uint4v{0u, 0u, 0u, 0u};
            r.hi[rt] = uint2v{0u, 0u};
        }
    }
}

// copy one 64 KiB stage: every wave copies 16 KiB as 16 wave-wide 1 KiB direct-to-LDS loads
__device__ __forceinline__ void stage_copy(const uint8_t *__restrict__ src, uint8_t *lds_dst, int wave, int lane)
{
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int blk = wave * 16 + u;  // 1 KiB block index inside the stage
        __builtin_amdgcn_global_load_lds((glb_u32 *)(src + (size_t)blk * 1024 + lane * 16),
                                         (lds_u32 *)(lds_dst + blk * 1024), 16, 0, 0);
    }
}

template <int BITS, int D>
__device__ __forceinline__ void gemm_word(const GemmTileRegs<BITS> &r, const HighBits (&hb)[kGemmRowTiles],
                                          const RowTables (&tb)[kGemmRowTiles], const uint8_t *stage, int boff,
                                          float4v (&acc)[kGemmRowTiles][kGemmTokTiles])
{
    uint4v op[kGemmRowTiles][2];
#pragma unroll
    for (int rt = 0; rt < kGemmRowTiles; ++rt) decode_word<BITS, D>(r.lo[rt][D], hb[rt], tb[rt], op[rt][0], op[rt][1]);
#pragma unroll
    for (int a = 0; a < 2; ++a) {
        const int g = 2 * D + a;
#pragma unroll
        for (int mt = 0; mt < kGemmTokTiles; ++mt) {
            const uint4v b = *reinterpret_cast<const uint4v *>(stage + (mt * 8 + g) * 1024 + boff);
#pragma unroll
            for (int rt = 0; rt < kGemmRowTiles; ++rt)
                acc[rt][mt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op[rt][a]), as_half8(b), acc[rt][mt], 0, 0, 0);
        }
    }
}

template <int BITS>
__global__ void __launch_bounds__(kGemmWaves * 64, 1)
gemm_kernel(const uint8_t *__restrict__ packed, const uint8_t *__restrict__ lutB, const uint8_t *__restrict__ xs,
            uint16_t *__restrict__ y, int M, int Mpad, int N, int K)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];  // 2 stages x 64 KiB

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int q = lane >> 4, j = lane & 15, bq = lane >> 4;
    const int kc = K / kTileCols, nt = N / kTileRows;
    const int t0 = (blockIdx.x * kGemmWaves + wave) * kGemmRowTiles;   // first row tile of this wave
    const int mt0 = blockIdx.y * kGemmTokTiles;                        // first token tile of this workgroup
    const int boff = (j * 4 + q) * 16;                                  // lane's 16 bytes inside a 1 KiB operand block

    // activations of chunk c for this workgroup's 128 tokens: one contiguous 64 KiB block
    const size_t chunk_stride = (size_t)(Mpad >> 4) * 8 * 1024;
    const uint8_t *xs_base = xs + (size_t)mt0 * 8 * 1024;

    RowTables tb[kGemmRowTiles];
#pragma unroll
    for (int rt = 0; rt < kGemmRowTiles; ++rt) {
        const int row = min((t0 + rt), nt - 1) * kTileRows + (lane & 15);
        if (BITS == 2) {
            const uint2v v = *reinterpret_cast<const uint2v *>(lutB + (size_t)row * 8);
            tb[rt].lo[0] = v[0]; tb[rt].hi[0] = v[1]; tb[rt].lo[1] = 0; tb[rt].hi[1] = 0;
        } else {
            const uint4v v = *reinterpret_cast<const uint4v *>(lutB + (size_t)row * 16);
            tb[rt].lo[0] = v[0]; tb[rt].lo[1] = v[1]; tb[rt].hi[0] = v[2]; tb[rt].hi[1] = v[3];
        }
    }

    float4v acc[kGemmRowTiles][kGemmTokTiles];
#pragma unroll
    for (int rt = 0; rt < kGemmRowTiles; ++rt)
#pragma unroll
        for (int mt = 0; mt < kGemmTokTiles; ++mt) acc[rt][mt] = float4v{0.f, 0.f, 0.f, 0.f};

    GemmTileRegs<BITS> r0, r1;
    load_gemm_tiles<BITS>(r0, packed, t0, nt, kc, 0, lane);
    stage_copy(xs_base, lds, wave, lane);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    auto compute = [&](const GemmTileRegs<BITS> &r, const uint8_t *stage) {
        HighBits hb[kGemmRowTiles];
#pragma unroll
        for (int rt = 0; rt < kGemmRowTiles; ++rt) {
            hb[rt] = HighBits{0u, 0u};
            if (BITS == 3) hb[rt] = regroup_high(r.hi[rt]);
        }
        gemm_word<BITS, 0>(r, hb, tb, stage, boff, acc);
        gemm_word<BITS, 1>(r, hb, tb, stage, boff, acc);
        gemm_word<BITS, 2>(r, hb, tb, stage, boff, acc);
        gemm_word<BITS, 3>(r, hb, tb, stage, boff, acc);
    };

    for (int c = 0; c < kc; c += 2) {
        // even chunk: compute from stage 0 / r0 while chunk c+1 lands in stage 1 / r1
        if (c + 1 < kc) {
            load_gemm_tiles<BITS>(r1, packed, t0, nt, kc, c + 1, lane);
            stage_copy(xs_base + (size_t)(c + 1) * chunk_stride, lds + kStageBytes, wave, lane);
        }
        compute(r0, lds);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (c + 1 >= kc) break;
        if (c + 2 < kc) {
            load_gemm_tiles<BITS>(r0, packed, t0, nt, kc, c + 2, lane);
            stage_copy(xs_base + (size_t)(c + 2) * chunk_stride, lds, wave, lane);
        }
        compute(r1, lds + kStageBytes);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
    }

    // store: lane (bq, j) holds rows 4bq..4bq+3 of token 16*mt + j
#pragma unroll
    for (int rt = 0; rt < kGemmRowTiles; ++rt) {
        if (t0 + rt >= nt) continue;
#pragma unroll
        for (int mt = 0; mt < kGemmTokTiles; ++mt) {
            const int m = (mt0 + mt) * 16 + j;
            if (m < M) {
                typedef _Float16 half4 __attribute__((ext_vector_type(4)));
                half4 o;
#pragma unroll
                for (int u = 0; u < 4; ++u) o[u] = (_Float16)acc[rt][mt][u];
                *reinterpret_cast<half4 *>(y + (size_t)m * N + (size_t)(t0 + rt) * kTileRows + 4 * bq) = o;
            }
        }
    }
}

int launch_gemm(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, void *workspace, const GemmPlan &plan, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    const int Mpad = plan.m_pad;
    if (int e = launch_smooth(x, s, workspace, M, Mpad, K, 1, stream)) return e;
    const uint8_t *lutB = static_cast<const uint8_t *>(lut) + (size_t)N * (bits == 2 ? 4 : 8) * 4;
    const int nt = N / kTileRows;
    const int rows_per_wg = kGemmWaves * kGemmRowTiles;
    const dim3 grid((nt + rows_per_wg - 1) / rows_per_wg, Mpad / kGemmTokens), block(kGemmWaves * 64);
    const size_t lds_bytes = 2 * kStageBytes;
    static bool attr_set[2] = {false, false};
    if (bits == 2) {
        if (!attr_set[0]) {
            if (hipError_t e = hipFuncSetAttribute((const void *)gemm_kernel<2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes)) return (int)e;
            attr_set[0] = true;
        }
        hipLaunchKernelGGL(gemm_kernel<2>, grid, block, lds_bytes, stream, (const uint8_t *)packed, lutB,
                           (const uint8_t *)workspace, y, M, Mpad, N, K);
    } else {
        if (!attr_set[1]) {
            if (hipError_t e = hipFuncSetAttribute((const void *)gemm_kernel<3>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes)) return (int)e;
            attr_set[1] = true;
        }
        hipLaunchKernelGGL(gemm_kernel<3>, grid, block, lds_bytes, stream, (const uint8_t *)packed, lutB,
                           (const uint8_t *)workspace, y, M, Mpad, N, K);
    }
    return (int)hipGetLastError();
}

}  // namespace lcd
