// Clustering-side kernels that need no calibration data (gfx950): nearest-centroid assignment of
// dense fp16 weights (the state the reclassification rule of paper Sec. 3.2, Eq. 6 maintains),
// cluster sizes, and the merge of the two closest centroids (Sec. 3.3, Eq. 8).  All of them stream
// the matrix once; none is a contraction, so there is no matrix-core work here.
#include <hip/hip_runtime.h>
#include "lcd_internal.h"
#include "lcd_device.h"

namespace lcd {

constexpr int kAssignThreads = 256;
constexpr int kAssignCols = kAssignThreads * 8;   // columns of a row per pass of its workgroup

__device__ __forceinline__ double half_bits_to_double(uint16_t b) { return (double)(float)__builtin_bit_cast(_Float16, b); }

// neighbours of an fp16 value in the order of the reals (bit patterns; -0 counts as 0)
__device__ __forceinline__ uint16_t half_next_up(uint16_t b)
{
    if ((b & 0x7fffu) == 0) return 0x0001u;
    return (b & 0x8000u) ? (uint16_t)(b - 1) : (uint16_t)(b + 1);
}
__device__ __forceinline__ uint16_t half_next_down(uint16_t b)
{
    if ((b & 0x7fffu) == 0) return 0x8001u;
    return (b & 0x8000u) ? (uint16_t)(b + 1) : (uint16_t)(b - 1);
}

// ---- nearest centroid ------------------------------------------------------------------------
// With ascending centroids the nearest one is found by counting the boundaries (c_i + c_i+1)/2
// a weight lies strictly above (a weight ON a boundary stays with the lower centroid).  A boundary
// need not be an fp16 number, but "w > boundary" for an fp16 w is the same as "w >= u" with u the
// smallest fp16 number above the boundary; u is found once per row in fp64, where the boundary is
// exact, and the per-weight comparisons are exact fp32 ones.
template <int NTHR>   // boundaries the container can have: 3, 7 or 15
__global__ void __launch_bounds__(kAssignThreads) assign_kernel(const uint16_t *__restrict__ w, const uint16_t *__restrict__ codebook,
                                                                uint8_t *__restrict__ idx, int K, int ncent)
{
    __shared__ float thr[16];
    const int n = blockIdx.x;          // rows on the x axis: N may exceed the y limit of a grid
    if (threadIdx.x < NTHR) {
        float u = 0.0f;
        if ((int)threadIdx.x + 1 < ncent) {
            const uint16_t *row = codebook + (size_t)n * (NTHR + 1);
            const double m = 0.5 * (half_bits_to_double(row[threadIdx.x]) + half_bits_to_double(row[threadIdx.x + 1]));   // exact
            uint16_t h = __builtin_bit_cast(uint16_t, (_Float16)(float)m);   // within an fp16 step or two of m
#pragma unroll
            for (int it = 0; it < 3; ++it) {          // walk down while the lower neighbour is still above m
                const uint16_t d = half_next_down(h);
                if (half_bits_to_double(d) > m) h = d;
            }
#pragma unroll
            for (int it = 0; it < 3; ++it)            // walk up while h is not above m (stops at infinity)
                if (!(half_bits_to_double(h) > m) && (h & 0x7fffu) != 0x7c00u) h = half_next_up(h);
            u = (float)__builtin_bit_cast(_Float16, h);
        }
        thr[threadIdx.x] = u;
    }
    __syncthreads();
    // the workgroup walks its row: the boundaries are found once per row
    for (int k0 = (int)threadIdx.x * 8; k0 < K; k0 += kAssignCols) {   // K is a multiple of 256: 8 columns are all inside or all outside
        const uint4v v = stream_load(reinterpret_cast<const uint4v *>(w + (size_t)n * K + k0));
        float wf[8];
        uint32_t cnt[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            wf[e] = (float)__builtin_bit_cast(_Float16, (uint16_t)(v[e >> 1] >> (16 * (e & 1))));
            cnt[e] = 0;
        }
#pragma unroll
        for (int i = 0; i < NTHR; ++i) {
            if (i + 1 >= ncent) break;     // uniform
            const float t = thr[i];
#pragma unroll
            for (int e = 0; e < 8; ++e) cnt[e] += wf[e] >= t ? 1u : 0u;
        }
        uint2v o;
        o[0] = cnt[0] | (cnt[1] << 8) | (cnt[2] << 16) | (cnt[3] << 24);
        o[1] = cnt[4] | (cnt[5] << 8) | (cnt[6] << 16) | (cnt[7] << 24);
        stream_store(reinterpret_cast<uint2v *>(idx + (size_t)n * K + k0), o);
    }
}

// ---- cluster sizes: one wave per row, one private LDS counter per (bin, lane) ---------------------
__global__ void __launch_bounds__(256) counts_kernel(const uint8_t *__restrict__ idx, uint32_t *__restrict__ counts, int N, int K, int slots)
{
    __shared__ uint32_t hist[4][16][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = (int)blockIdx.x * 4 + wave;     // N is a multiple of 16: every wave has a row
#pragma unroll
    for (int b = 0; b < 16; ++b) hist[wave][b][lane] = 0;
    const uint8_t *row = idx + (size_t)n * K;
    for (int k = lane * 16; k < K; k += 64 * 16) {
        const uint4v v = *reinterpret_cast<const uint4v *>(row + k);
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const uint32_t bin = (v[e >> 2] >> (8 * (e & 3))) & 15u;
            hist[wave][bin][lane] += 1;          // private to this lane: no atomics needed
        }
    }
    for (int b = 0; b < slots; ++b) {
        uint32_t c = hist[wave][b][lane];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) c += __shfl_down(c, off);
        if (lane == 0) counts[(size_t)n * slots + b] = c;
    }
}

// ---- merge decision: one thread per row ------------------------------------------------------------
// The pair with the smallest gap (gaps are exact in fp64; the lowest pair on equal gaps) becomes the
// mean of the two weighted by their cluster sizes, correctly rounded to fp16 (ties to even).  A finite
// fp16 number is an integer multiple of 2^-24 below 2^41 in magnitude and a cluster size is below 2^32,
// so the mean is the ratio of two integers, num / den with |num| < 2^75 and den < 2^34, and "which of
// two neighbouring fp16 numbers is nearer" is an integer comparison: no rounding happens anywhere.
struct U128 { uint64_t hi, lo; };
__device__ __forceinline__ U128 mul_64x64(uint64_t a, uint64_t b) { return U128{__umul64hi(a, b), a * b}; }
__device__ __forceinline__ U128 add128(U128 a, U128 b) { const uint64_t lo = a.lo + b.lo; return U128{a.hi + b.hi + (lo < a.lo ? 1u : 0u), lo}; }
__device__ __forceinline__ U128 sub128(U128 a, U128 b) { return U128{a.hi - b.hi - (a.lo < b.lo ? 1u : 0u), a.lo - b.lo}; }   // a >= b
__device__ __forceinline__ int cmp128(U128 a, U128 b) { return a.hi != b.hi ? (a.hi < b.hi ? -1 : 1) : (a.lo != b.lo ? (a.lo < b.lo ? -1 : 1) : 0); }

// magnitude of a finite fp16 bit pattern in units of 2^-24 (monotone in the 15-bit pattern)
__device__ __forceinline__ uint64_t half_units(uint32_t h15)
{
    const uint32_t e = h15 >> 10, f = h15 & 1023u;
    return e == 0 ? (uint64_t)f : (uint64_t)(1024u + f) << (e - 1);
}

// fp16 bit pattern nearest to (na * a + nb * b) / (na + nb), ties to even; (a + b) / 2 if na = nb = 0
__device__ uint16_t weighted_mean_half(uint16_t a, uint16_t b, uint32_t na, uint32_t nb)
{
    if (na == 0 && nb == 0) na = nb = 1;
    const U128 pa = mul_64x64(half_units(a & 0x7fffu), na), pb = mul_64x64(half_units(b & 0x7fffu), nb);
    const bool sa = (a & 0x8000u) != 0, sb = (b & 0x8000u) != 0;
    U128 num;
    bool neg;
    if (sa == sb) { num = add128(pa, pb); neg = sa; }
    else if (cmp128(pa, pb) >= 0) { num = sub128(pa, pb); neg = sa; }
    else { num = sub128(pb, pa); neg = sb; }
    const uint64_t den = (uint64_t)na + nb;
    // largest pattern h with units(h) * den <= num (the mean lies between the two centroids: h <= 0x7bff)
    uint32_t lo = 0, hi = 0x7bffu;
    while (lo < hi) {
        const uint32_t mid = (lo + hi + 1) >> 1;
        if (cmp128(mul_64x64(half_units(mid), den), num) <= 0) lo = mid; else hi = mid - 1;
    }
    uint32_t h = lo;
    if (h < 0x7bffu) {   // nearer of h and h + 1: 2 * num against (units(h) + units(h + 1)) * den
        const U128 twice = add128(num, num);
        const int c = cmp128(twice, mul_64x64(half_units(h) + half_units(h + 1), den));
        if (c > 0 || (c == 0 && (h & 1u))) ++h;
    }
    if (num.hi == 0 && num.lo == 0) neg = false;   // a mean of exactly zero is +0; a negative one that rounds to zero keeps its sign
    return (uint16_t)(h | (neg ? 0x8000u : 0u));
}

__global__ void __launch_bounds__(256) merge_kernel(const uint16_t *__restrict__ cb_in, const uint32_t *__restrict__ counts,
                                                    uint16_t *__restrict__ cb_out, uint8_t *__restrict__ merged, int N, int ncent, int slots)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    const uint16_t *src = cb_in + (size_t)n * slots;
    int a = 0;
    double best = half_bits_to_double(src[1]) - half_bits_to_double(src[0]);
    for (int i = 1; i + 1 < ncent; ++i) {
        const double g = half_bits_to_double(src[i + 1]) - half_bits_to_double(src[i]);
        if (g < best) { best = g; a = i; }
    }
    const uint16_t nc = weighted_mean_half(src[a], src[a + 1], counts[(size_t)n * slots + a], counts[(size_t)n * slots + a + 1]);
    uint16_t *dst = cb_out + (size_t)n * slots;
    for (int i = 0; i < slots; ++i) {
        uint16_t v = 0;
        if (i < a) v = src[i];
        else if (i == a) v = nc;
        else if (i < ncent - 1) v = src[i + 1];
        dst[i] = v;
    }
    merged[n] = (uint8_t)a;
}

// ---- re-numbering after a merge: idx' = idx - (idx > a), four indices per 32-bit operation -------
__global__ void __launch_bounds__(256) remap_kernel(const uint8_t *__restrict__ idx, const uint8_t *__restrict__ merged,
                                                    uint8_t *__restrict__ out, int K)
{
    const int n = blockIdx.x;
    const int k0 = ((int)blockIdx.y * 256 + (int)threadIdx.x) * 16;
    if (k0 >= K) return;
    const uint32_t bias = (127u - merged[n]) * 0x01010101u;     // byte + bias has bit 7 set iff byte > a (bytes < 16)
    const uint4v v = stream_load(reinterpret_cast<const uint4v *>(idx + (size_t)n * K + k0));
    uint4v o;
#pragma unroll
    for (int d = 0; d < 4; ++d) o[d] = v[d] - (((v[d] + bias) >> 7) & 0x01010101u);
    stream_store(reinterpret_cast<uint4v *>(out + (size_t)n * K + k0), o);
}

int launch_assign(const uint16_t *w, const uint16_t *codebook, int ncent, int N, int K, int bits, uint8_t *idx, void *stream)
{
    const dim3 grid((unsigned)N), block(kAssignThreads);
    if (bits == 2) hipLaunchKernelGGL(assign_kernel<3>, grid, block, 0, (hipStream_t)stream, w, codebook, idx, K, ncent);
    else if (bits == 3) hipLaunchKernelGGL(assign_kernel<7>, grid, block, 0, (hipStream_t)stream, w, codebook, idx, K, ncent);
    else hipLaunchKernelGGL(assign_kernel<15>, grid, block, 0, (hipStream_t)stream, w, codebook, idx, K, ncent);
    return (int)hipGetLastError();
}

int launch_counts(const uint8_t *idx, int N, int K, int bits, uint32_t *counts, void *stream)
{
    hipLaunchKernelGGL(counts_kernel, dim3((unsigned)(N / 4)), dim3(256), 0, (hipStream_t)stream, idx, counts, N, K, 1 << bits);
    return (int)hipGetLastError();
}

int launch_merge(const uint16_t *cb_in, const uint32_t *counts, const uint8_t *idx_in, int ncent, int N, int K, int bits,
                 uint16_t *cb_out, uint8_t *idx_out, uint8_t *merged, void *stream)
{
    hipLaunchKernelGGL(merge_kernel, dim3((unsigned)((N + 255) / 256)), dim3(256), 0, (hipStream_t)stream, cb_in, counts, cb_out, merged,
                       N, ncent, 1 << bits);
    if (hipError_t e = hipGetLastError()) return (int)e;
    hipLaunchKernelGGL(remap_kernel, dim3((unsigned)N, (unsigned)((K + 4095) / 4096)), dim3(256), 0, (hipStream_t)stream, idx_in, merged,
                       idx_out, K);
    return (int)hipGetLastError();
}

}  // namespace lcd
