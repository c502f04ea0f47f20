// Offline kernels: index packing / unpacking and table build, and the activation smoothing
// kernel of the prefill path.  Layout: see include/lcd.h.
#include <hip/hip_runtime.h>
#include "lcd_internal.h"
#include "lcd_device.h"

namespace lcd {

// ---- pack: one thread per (tile, lane); reads the lane's 64 index bytes, writes its words ----
template <int BITS>
__global__ void __launch_bounds__(256) pack_kernel(const uint8_t *__restrict__ idx, uint8_t *__restrict__ packed,
                                                   int N, int K, long long total)
{
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= total) return;
    const int kc = K / kTileCols;
    const int l = (int)(g & 63);
    const long long tile = g >> 6;
    const int c = (int)(tile % kc);
    const long long t = tile / kc;
    const int q = l >> 4, i = l & 15;
    const uint4v *src = reinterpret_cast<const uint4v *>(idx + (size_t)(t * kTileRows + i) * K + (size_t)c * kTileCols + q * kLaneCols);
    uint32_t lo[4] = {0, 0, 0, 0}, hi[4] = {0, 0, 0, 0};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        const uint4v v = src[d];  // 16 indices, one per byte
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t word = v[j];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int e16 = 4 * j + b;                 // position inside this group of 16
                const uint32_t val = (word >> (8 * b)) & ((1u << BITS) - 1u);
                lo[d] |= (val & 3u) << (2 * e16);
                if (BITS == 3) {
                    const int a = e16 >> 3, e = e16 & 7;
                    const int bit = 8 * ((e >> 2) + 2 * (e & 1)) + 2 * d + ((e & 3) >> 1);
                    hi[a] |= (val >> 2) << bit;
                }
                if (BITS == 4) hi[d] |= (val >> 2) << (2 * e16);
            }
        }
    }
    uint8_t *tile_ptr = packed + (size_t)tile * (kTileRows * kTileCols * BITS / 8);
    uint4v o = {lo[0], lo[1], lo[2], lo[3]};
    *reinterpret_cast<uint4v *>(tile_ptr + 16 * l) = o;
    if (BITS == 3) {
        uint2v h = {hi[0], hi[1]};
        *reinterpret_cast<uint2v *>(tile_ptr + 1024 + 8 * l) = h;
    }
    if (BITS == 4) {
        uint4v h = {hi[0], hi[1], hi[2], hi[3]};
        *reinterpret_cast<uint4v *>(tile_ptr + 1024 + 16 * l) = h;
    }
}

template <int BITS>
__global__ void __launch_bounds__(256) unpack_kernel(const uint8_t *__restrict__ packed, uint8_t *__restrict__ idx,
                                                     int N, int K, long long total)
{
    const long long g = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= total) return;
    const int kc = K / kTileCols;
    const int l = (int)(g & 63);
    const long long tile = g >> 6;
    const int c = (int)(tile % kc);
    const long long t = tile / kc;
    const int q = l >> 4, i = l & 15;
    const uint8_t *tile_ptr = packed + (size_t)tile * (kTileRows * kTileCols * BITS / 8);
    const uint4v lo = *reinterpret_cast<const uint4v *>(tile_ptr + 16 * l);
    uint2v hi = {0, 0};
    uint4v hi4 = {0, 0, 0, 0};
    if (BITS == 3) hi = *reinterpret_cast<const uint2v *>(tile_ptr + 1024 + 8 * l);
    if (BITS == 4) hi4 = *reinterpret_cast<const uint4v *>(tile_ptr + 1024 + 16 * l);
    uint4v *dst = reinterpret_cast<uint4v *>(idx + (size_t)(t * kTileRows + i) * K + (size_t)c * kTileCols + q * kLaneCols);
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        uint4v out;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            uint32_t word = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                const int e16 = 4 * j + b;
                uint32_t val = (lo[d] >> (2 * e16)) & 3u;
                if (BITS == 3) {
                    const int a = e16 >> 3, e = e16 & 7;
                    const int bit = 8 * ((e >> 2) + 2 * (e & 1)) + 2 * d + ((e & 3) >> 1);
                    val |= ((hi[a] >> bit) & 1u) << 2;
                }
                if (BITS == 4) val |= ((hi4[d] >> (2 * e16)) & 3u) << 2;
                word |= val << (8 * b);
            }
            out[j] = word;
        }
        dst[d] = out;
    }
}

// ---- table build: one thread per output row -----------------------------------------------
// Section A (fp32, accumulator order): element ((n/4)*NC + j)*4 + n%4, NC = 4 (2 bits) or 8.
//   2 bits: A[j] = C[n][j].   3 bits: A[j] = (C[n][j] + C[n][4+j])/2, A[4+j] = (C[n][j] - C[n][4+j])/2,
//   so that C[n][4h+l] = A[l] + (1-2h) * A[4+l].
// Section B (byte-split tables for v_perm_b32), starting at byte N*NC*4:
//   2 bits: per row {low bytes of C[n][0..3], high bytes of C[n][0..3]}            (8 bytes)
//   3 bits: per row {low 0..3, low 4..7, high 0..3, high 4..7}                      (16 bytes)
// 4 bits: no section A (the single-token case runs on the register dequantiser too); per row
//   {low bytes of C[n][0..15], high bytes of C[n][0..15]}                                      (32 bytes)
template <int BITS>
__global__ void __launch_bounds__(256) build_lut_kernel(const uint16_t *__restrict__ codebook, uint8_t *__restrict__ lut, int N)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    constexpr int NCENT = 1 << BITS;
    constexpr int NC = BITS == 2 ? 4 : 8;
    uint16_t c[NCENT];
#pragma unroll
    for (int j = 0; j < NCENT; ++j) c[j] = codebook[(size_t)n * NCENT + j];
    if (BITS == 4) {
        uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            w[j >> 2] |= (uint32_t)(c[j] & 255) << (8 * (j & 3));
            w[4 + (j >> 2)] |= (uint32_t)(c[j] >> 8) << (8 * (j & 3));
        }
        uint4v *dst = reinterpret_cast<uint4v *>(lut) + 2 * (size_t)n;
        dst[0] = uint4v{w[0], w[1], w[2], w[3]};
        dst[1] = uint4v{w[4], w[5], w[6], w[7]};
        return;
    }
    float *secA = reinterpret_cast<float *>(lut);
    const size_t baseA = (size_t)(n >> 2) * NC * 4 + (n & 3);
    if (BITS == 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) secA[baseA + 4 * j] = (float)__builtin_bit_cast(_Float16, c[j]);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float c0 = (float)__builtin_bit_cast(_Float16, c[j]);
            const float c1 = (float)__builtin_bit_cast(_Float16, c[4 + j]);
            secA[baseA + 4 * j] = 0.5f * (c0 + c1);
            secA[baseA + 4 * (4 + j)] = 0.5f * (c0 - c1);
        }
    }
    uint32_t *secB = reinterpret_cast<uint32_t *>(lut + (size_t)N * NC * 4);
    if (BITS == 2) {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) { lo |= (uint32_t)(c[j] & 255) << (8 * j); hi |= (uint32_t)(c[j] >> 8) << (8 * j); }
        secB[2 * (size_t)n] = lo;
        secB[2 * (size_t)n + 1] = hi;
    } else {
        uint32_t lo0 = 0, lo1 = 0, hi0 = 0, hi1 = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            lo0 |= (uint32_t)(c[j] & 255) << (8 * j);      hi0 |= (uint32_t)(c[j] >> 8) << (8 * j);
            lo1 |= (uint32_t)(c[4 + j] & 255) << (8 * j);  hi1 |= (uint32_t)(c[4 + j] >> 8) << (8 * j);
        }
        uint4v o = {lo0, lo1, hi0, hi1};
        reinterpret_cast<uint4v *>(secB)[n] = o;
    }
}

// ---- activation smoothing: xs[m][k] = fp16( x[m][k] / s[k] )  (paper Sec. 3.4) -------------
// Prefill path only (the decode kernels smooth in place).  Output: operand order of
// v_mfma_f32_32x32x16_f16,
//   [chunk k/256][token block m/32][half (k%256)/128][step g=(k%64)/8][(k%128)/64][m%32][8 slots],
// inside a group of 8 the slot order 0,4,1,5,2,6,3,7 that the register dequantiser produces;
// tokens padded with zeros up to Mpad (a multiple of 128).
// One workgroup per (chunk, token block): 32 tokens x 256 columns = 16 KiB in, 16 KiB out, both
// contiguous per row / per block.  Rows are read coalesced (32 threads per 512-byte row), each
// thread smooths 8 values, and the tile is turned into operand order through LDS so that the
// stores are coalesced too (16-byte stores scattered 1 KiB apart ran at a third of the rate).
constexpr int kSmoothRowBytes = 32 * 16 + 16;   // one [m 32][16 B] row of the tile in LDS, padded
// s_q != 0: the input transformation of Sec. 4.1 (Eq. 10-11) instead -- the activations leave as INT8 codes
// (integers up to 128 in magnitude, exact as fp16 numbers); the divisor-only part of the division is
// shared by the thread's four token rows.
__device__ __forceinline__ void smooth_tile(const uint16_t *__restrict__ x, const float *__restrict__ s,
                                            _Float16 *__restrict__ xs, int M, int Mpad, int K, int c, int mb, float s_q)
{
    __shared__ __attribute__((aligned(16))) uint8_t tile[32 * kSmoothRowBytes];
    const int t = threadIdx.x;
    // a thread's four groups are the same 8 columns of four token rows: one set of reciprocals
    const int kg = t & 31, k = c * kTileCols + 8 * kg;
    const bool quantised = s_q != 0.0f;   // uniform
    float r[8];
    Divisor dv[8];
    {
        const float4v s0 = *reinterpret_cast<const float4v *>(s + k);
        const float4v s1 = *reinterpret_cast<const float4v *>(s + k + 4);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float se = e < 4 ? s0[e] : s1[e - 4];
            r[e] = __builtin_amdgcn_rcpf(se);
            dv[e] = make_divisor(se, quantised ? s_q : 1.0f);
        }
    }
    uint4v xin[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {               // all four loads in flight together
        const int m = mb * 32 + ((t + 256 * u) >> 5);
        xin[u] = uint4v{0u, 0u, 0u, 0u};
        if (m < M) xin[u] = stream_load(reinterpret_cast<const uint4v *>(x + (size_t)m * K + k));   // read once
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int grp = t + 256 * u;            // input order: 32 groups of 8 columns per token row
        const int ml = grp >> 5;
        const int m = mb * 32 + ml;
        half8 o;
        if (m < M) {
            const uint4v xv = xin[u];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint16_t xb = (uint16_t)(xv[e >> 1] >> (16 * (e & 1)));
                const int slot = e < 4 ? 2 * e : 2 * (e - 4) + 1;
                o[slot] = quantised ? quantise_one(xb, dv[e]) : smooth_with(xb, r[e]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (_Float16)0.0f;
        }
        const int h = kg >> 4, kh = (kg >> 3) & 1, g = kg & 7;
        const int row = (h * 8 + g) * 2 + kh;   // position of this group of 8 columns in operand order
        *reinterpret_cast<half8 *>(tile + row * kSmoothRowBytes + ml * 16) = o;
    }
    __syncthreads();
    _Float16 *dst = xs + ((size_t)c * (Mpad >> 5) + mb) * (32 * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int grp = t + 256 * u;            // output order: [row 32][m 32] groups of 8 halfs
        const int row = grp >> 5, ml = grp & 31;
        *reinterpret_cast<half8 *>(dst + (size_t)grp * 8) = *reinterpret_cast<const half8 *>(tile + row * kSmoothRowBytes + ml * 16);
    }
}

__global__ void __launch_bounds__(256) smooth_kernel(const uint16_t *__restrict__ x, const float *__restrict__ s,
                                                     _Float16 *__restrict__ xs, int M, int Mpad, int K, float s_q)
{
    smooth_tile(x, s, xs, M, Mpad, K, blockIdx.x, blockIdx.y, s_q);
}

// the activations of several layers in one launch: grid.z = layer, grid.x = the widest layer's chunks
struct SmoothBatch { SmoothItem p[kMaxGroup]; };
__global__ void __launch_bounds__(256) smooth_group_kernel(const SmoothBatch batch, int M, int Mpad)
{
    const SmoothItem it = batch.p[blockIdx.z];
    if ((int)blockIdx.x * kTileCols >= it.K) return;   // uniform over the workgroup
    smooth_tile(it.x, it.s, (_Float16 *)it.xs, M, Mpad, it.K, blockIdx.x, blockIdx.y, it.s_q);
}

int launch_smooth_group(const SmoothItem *items, int count, int M, int Mpad, void *stream)
{
    SmoothBatch batch{};
    int widest = 0;
    for (int i = 0; i < count; ++i) { batch.p[i] = items[i]; widest = items[i].K > widest ? items[i].K : widest; }
    const dim3 grid((unsigned)(widest / kTileCols), (unsigned)(Mpad / 32), (unsigned)count), block(256);
    hipLaunchKernelGGL(smooth_group_kernel, grid, block, 0, (hipStream_t)stream, batch, M, Mpad);
    return (int)hipGetLastError();
}

int launch_smooth(const uint16_t *x, const float *s, void *xs, int M, int Mpad, int K, float s_q, void *stream)
{
    const dim3 grid((unsigned)(K / kTileCols), (unsigned)(Mpad / 32)), block(256);
    hipLaunchKernelGGL(smooth_kernel, grid, block, 0, (hipStream_t)stream, x, s, (_Float16 *)xs, M, Mpad, K, s_q);
    return (int)hipGetLastError();
}

int launch_pack(const uint8_t *idx, int N, int K, int bits, void *packed, void *stream)
{
    const long long total = (long long)(N / kTileRows) * (K / kTileCols) * 64;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (bits == 2) hipLaunchKernelGGL(pack_kernel<2>, grid, block, 0, (hipStream_t)stream, idx, (uint8_t *)packed, N, K, total);
    else if (bits == 3) hipLaunchKernelGGL(pack_kernel<3>, grid, block, 0, (hipStream_t)stream, idx, (uint8_t *)packed, N, K, total);
    else hipLaunchKernelGGL(pack_kernel<4>, grid, block, 0, (hipStream_t)stream, idx, (uint8_t *)packed, N, K, total);
    return (int)hipGetLastError();
}

int launch_unpack(const void *packed, int N, int K, int bits, uint8_t *idx, void *stream)
{
    const long long total = (long long)(N / kTileRows) * (K / kTileCols) * 64;
    const dim3 grid((unsigned)((total + 255) / 256)), block(256);
    if (bits == 2) hipLaunchKernelGGL(unpack_kernel<2>, grid, block, 0, (hipStream_t)stream, (const uint8_t *)packed, idx, N, K, total);
    else if (bits == 3) hipLaunchKernelGGL(unpack_kernel<3>, grid, block, 0, (hipStream_t)stream, (const uint8_t *)packed, idx, N, K, total);
    else hipLaunchKernelGGL(unpack_kernel<4>, grid, block, 0, (hipStream_t)stream, (const uint8_t *)packed, idx, N, K, total);
    return (int)hipGetLastError();
}

int launch_build_lut(const uint16_t *codebook, int N, int bits, void *lut, void *stream)
{
    const dim3 grid((unsigned)((N + 255) / 256)), block(256);
    if (bits == 2) hipLaunchKernelGGL(build_lut_kernel<2>, grid, block, 0, (hipStream_t)stream, codebook, (uint8_t *)lut, N);
    else if (bits == 3) hipLaunchKernelGGL(build_lut_kernel<3>, grid, block, 0, (hipStream_t)stream, codebook, (uint8_t *)lut, N);
    else hipLaunchKernelGGL(build_lut_kernel<4>, grid, block, 0, (hipStream_t)stream, codebook, (uint8_t *)lut, N);
    return (int)hipGetLastError();
}

const char *hip_error_name(int err) { return hipGetErrorString((hipError_t)err); }

}  // namespace lcd
