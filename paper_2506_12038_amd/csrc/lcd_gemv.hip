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

// ---- single-token bucket kernel: persistent workgroups over a group of layers ---------------
//
// The host gives every layer of the group a number of workgroups proportional to its work; a
// workgroup owns a contiguous run of row tiles of ONE layer and walks it in "visits" of up to
// kVisitTiles row tiles.  Per visit:
//   prologue   smoothed activations of the layer (all K, first visit only) and the visit's
//              per-bucket multipliers go to LDS; one barrier;
//   segments   the 8 waves split K into segments of 16 chunks (two 256-column chunks per wave).
//              For each segment a wave loads its activations LDS -> registers once, then streams
//              the visit's row tiles: 2-3 KiB of packed indices per tile, 16-32 sparse MFMAs,
//              and (once per 2 or 4 tiles) a few VALU ops that turn bucket sums into partial
//              outputs, which the wave adds into its own LDS slot (no synchronisation);
//   epilogue   one barrier; the workgroup adds the 8 waves' slots in a fixed order, stores y.
// Loads of packed indices run kSets-1 steps ahead of the arithmetic, across segment and visit
// boundaries.  Matrix and vector instructions of one SIMD do not overlap in time (measured), so
// the instruction count per byte is what matters, not the number of waves.
constexpr int kBW = 8;            // waves per workgroup
constexpr int kBCH = 2;           // chunks per wave per segment (their activations stay in registers)
constexpr int kBSeg = kBW * kBCH; // chunks per segment (one pass of the workgroup over K)
constexpr int kSets = 4;          // register sets in rotation (loads run kSets-1 steps ahead)
constexpr int kVisitTiles = 32;   // row tiles per visit

struct BucketProblem {
    const uint8_t *packed;
    const float *lutA;
    const uint16_t *x;
    const float *s;
    uint16_t *y;
    int nt, kc;
    int tiles_base, tiles_extra;  // workgroup i of this layer owns tiles_base (+1 if i < tiles_extra) row tiles
};
struct BucketBatch {
    BucketProblem p[kMaxGroup];
    int wg_begin[kMaxGroup + 1];  // first workgroup of every layer
    int count;
#ifdef LCD_TRACE
    unsigned long long *trace;   // debug builds only: 16 timestamps per workgroup
#endif
};
#ifdef LCD_TRACE
#define LCD_STAMP(slot) do { if (threadIdx.x == 0 && batch.trace) batch.trace[blockIdx.x * 16 + (slot)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define LCD_STAMP(slot) do { } while (0)
#endif

// Walks the (visit, segment, tile) sequence of one workgroup.  Everything is wave-uniform.
// Each (visit, segment) run is padded to a multiple of kSets steps so that the register-set
// rotation is static; padding steps load nothing and compute nothing.
struct Cursor {
    int v0, v1, range_end, sg, i, steps;
    bool done;
};

__device__ __forceinline__ int pad_sets(int n) { return (n + kSets - 1) / kSets * kSets; }

__device__ __forceinline__ void cursor_begin(Cursor &c, int ta, int tb)
{
    c.v0 = ta; c.range_end = tb; c.v1 = min(tb, ta + kVisitTiles);
    c.sg = 0; c.i = 0; c.steps = pad_sets(c.v1 - c.v0); c.done = ta >= tb;
}

__device__ __forceinline__ void cursor_next_visit(Cursor &c)
{
    c.sg = 0; c.i = 0;
    if (c.v1 < c.range_end) {
        c.v0 = c.v1; c.v1 = min(c.range_end, c.v0 + kVisitTiles); c.steps = pad_sets(c.v1 - c.v0);
    } else {
        c.done = true;
    }
}

__device__ __forceinline__ void cursor_advance(Cursor &c, int nseg)
{
    if (c.done) return;
    if (++c.i < c.steps) return;
    c.i = 0;
    if (++c.sg < nseg) return;
    cursor_next_visit(c);
}

template <int BITS>
struct StepRegs {
    uint4v lo[kBCH];   // the lane's 64 two-bit fields of this (tile, chunk)
    uint2v hi[kBCH];   // 3 bits only: its 64 third bits
};

template <int BITS>
__device__ __forceinline__ void issue_step_loads(StepRegs<BITS> &r, const Cursor &c, __amdgpu_buffer_rsrc_t rs, int kc, int wave, int lane)
{
    constexpr uint32_t TB = BITS == 2 ? 1024 : 1536;
    // a finished cursor or a padding step issues loads that are out of range: zeros, no traffic
    const int tile = c.v0 + c.i;
    const bool tv = !c.done && tile < c.v1;
#pragma unroll
    for (int ch = 0; ch < kBCH; ++ch) {
        const int chunk = c.sg * kBSeg + wave * kBCH + ch;
        const bool v = tv && chunk < kc;
        const uint32_t o = ((uint32_t)tile * (uint32_t)kc + (uint32_t)chunk) * TB;
        r.lo[ch] = __builtin_amdgcn_raw_buffer_load_b128(rs, v ? o + 16 * lane : kOob, 0, 0);
        if (BITS == 3) r.hi[ch] = __builtin_amdgcn_raw_buffer_load_b64(rs, v ? o + 1024 + 8 * lane : kOob, 0, 0);
    }
}

template <int BITS>
__global__ void __launch_bounds__(kBW * 64, 1) gemv_bucket_kernel(const BucketBatch batch)
{
    constexpr int NC = BITS == 2 ? 4 : 8;        // accumulator columns one row tile uses
    constexpr int TG = 16 / NC;                  // row tiles that share one reduction (4 or 2)
    constexpr uint32_t TB = BITS == 2 ? 1024 : 1536;
    constexpr int NT = kBW * 64;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS: [ xs: one segment, kBSeg*256 halfs ][ cf: kVisitTiles*16*NC floats ][ part: kBW*kVisitTiles*16 floats ]
    _Float16 *xs_lds = reinterpret_cast<_Float16 *>(smem);
    float *cf_lds = reinterpret_cast<float *>(smem + (size_t)kBSeg * kTileCols * 2);
    float *part = cf_lds + kVisitTiles * 16 * NC;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keeps addresses scalar
    const int q = lane >> 4, j = lane & 15, bq = lane >> 4;
    LCD_STAMP(0);

    // which layer, which row tiles
    int pi = 0;
    for (int i = 1; i < batch.count; ++i) pi += ((int)blockIdx.x >= batch.wg_begin[i]) ? 1 : 0;
    const BucketProblem pb = batch.p[pi];
    const int li = (int)blockIdx.x - batch.wg_begin[pi];
    const int ta = li * pb.tiles_base + min(li, pb.tiles_extra);
    const int tb = ta + pb.tiles_base + (li < pb.tiles_extra ? 1 : 0);
    const int kc = pb.kc, nseg = (kc + kBSeg - 1) / kBSeg;
    const __amdgpu_buffer_rsrc_t rs_packed = make_rsrc(pb.packed, (uint32_t)pb.nt * (uint32_t)kc * TB);
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(pb.x, (uint32_t)kc * kTileCols * 2);
    const __amdgpu_buffer_rsrc_t rs_s = make_rsrc(pb.s, (uint32_t)kc * kTileCols * 4);
    const __amdgpu_buffer_rsrc_t rs_lut = make_rsrc(pb.lutA, (uint32_t)pb.nt * 16 * NC * 4);

    Cursor pf{}, cur{};
    cursor_begin(pf, ta, tb);
    cur = pf;
    if (cur.done) return;

    // Activations.  A segment is kBSeg*256 = 8 * (threads of the workgroup) columns, and thread t of
    // wave w smooths columns [8t, 8t+8) of it -- which lie in wave w's own two chunks.  So a wave
    // stages its activations through its own 1 KiB of LDS (to fan 8 values out to the 16 lanes
    // that need them) without any workgroup synchronisation.  The loads for a segment are issued
    // one segment ahead; the very first ones head the kernel, before the tile loads, because they
    // start the longest dependency chain.  Reads past the end of x / s return zero through the
    // buffer resource.
    const int groups = kc * (kTileCols / 8);
    uint4v xv;
    float4v s0, s1;
    auto load_x = [&](int sg, bool valid) {
        const uint32_t g = (uint32_t)sg * NT + threadIdx.x;
        xv = __builtin_amdgcn_raw_buffer_load_b128(rs_x, valid ? g * 16 : kOob, 0, 0);
        s0 = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs_s, valid ? g * 32 : kOob, 0, 0));
        s1 = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs_s, valid ? g * 32 + 16 : kOob, 0, 0));
    };
    load_x(0, true);
    // multipliers of the first visit: (tiles * 4 * NC) float4, at most CFR per thread
    constexpr int CFR = kVisitTiles * 4 * NC / NT;
    static_assert(CFR * NT == kVisitTiles * 4 * NC, "multiplier preload must cover a full visit");
    const int nf4_first = (cur.v1 - cur.v0) * 4 * NC;
    uint4v cfv[CFR];
#pragma unroll
    for (int u = 0; u < CFR; ++u) {
        const int e = u * NT + (int)threadIdx.x;
        cfv[u] = __builtin_amdgcn_raw_buffer_load_b128(rs_lut, e < nf4_first ? ((uint32_t)cur.v0 * 4 * NC + e) * 16 : kOob, 0, 0);
    }
    StepRegs<BITS> r0, r1, r2, r3;
    issue_step_loads<BITS>(r0, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);

    uint4v A[kBCH][8];   // this wave's smoothed activations of the current segment, 8 operands per chunk
    half16 B1;        // constant routing matrix (index c -> column c), built after the prologue
    float *my_part = part + wave * (kVisitTiles * 16);
    LCD_STAMP(1);

    // bucket sums of one (tile, chunk): columns [0, NC) of a 16x16 accumulator
    auto tile_sums = [&](const StepRegs<BITS> &r) -> float4v {
        float4v accx = {0.f, 0.f, 0.f, 0.f}, accy = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ch = 0; ch < kBCH; ++ch) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int idxreg = (int)r.lo[ch][d];
                // half a = 0 uses index bits [15:0], a = 1 bits [31:16]
                if (BITS == 2) {
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d]), B1, accx, idxreg, 0, 0);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d + 1]), B1, accy, idxreg, 0, 1);
                } else {
                    // sign-flipped operands: pair v of half a has its two third bits 16 apart in word a
                    // of r.hi; one 64-bit shift moves them to bits 15 / 31 of both words, one
                    // xor-and per word applies them
                    const unsigned long long h64 = ((unsigned long long)r.hi[ch][1] << 32) | r.hi[ch][0];
                    uint4v f0, f1;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int sh = 15 - (8 * (v >> 1) + 2 * d + (v & 1));
                        unsigned long long t = h64;   // one full-rate v_lshlrev_b64 (the compiler would split it in two)
                        if (sh) asm("v_lshlrev_b64 %0, %1, %2" : "=v"(t) : "n"(sh), "v"(h64));
                        f0[v] = xor_and(A[ch][2 * d][v], (uint32_t)t, 0x80008000u);
                        f1[v] = xor_and(A[ch][2 * d + 1][v], (uint32_t)(t >> 32), 0x80008000u);
                    }
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d]), B1, accx, idxreg, 0, 0);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f0), B1, accy, idxreg, 0, 0);
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[ch][2 * d + 1]), B1, accx, idxreg, 0, 1);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f1), B1, accy, idxreg, 0, 1);
                }
            }
        }
        if (BITS == 2) return accx + accy;
        // 3 bits: the sign-flipped sums move from columns 0..3 to columns 4..7
        float4v m;
#pragma unroll
        for (int u = 0; u < 4; ++u) m[u] = accx[u] + dpp_f32<0x114>(accy[u]);   // row_shr:4
        return m;
    };

    // TG tiles share one multiply-and-reduce: tile u of the group moves to columns [u*NC, (u+1)*NC)
    auto reduce_group = [&](float4v m, int tl0) {
        const int tl = tl0 + j / NC;                    // this lane's tile inside the visit
        float4v cf = {0.f, 0.f, 0.f, 0.f};
        if (cur.v0 + tl < cur.v1) cf = *reinterpret_cast<const float4v *>(&cf_lds[((tl * 4 + bq) * NC + (j % NC)) * 4]);
        float4v pv;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v = m[u] * cf[u];
            v += dpp_f32<kDppQuadXor1>(v);
            v += dpp_f32<kDppQuadXor2>(v);
            if (NC == 8) v += dpp_f32<kDppRowHalfMirror>(v);
            pv[u] = v;
        }
        if ((j % NC) == 0 && cur.v0 + tl < cur.v1) {
            float4v *slot = reinterpret_cast<float4v *>(&my_part[tl * 16 + 4 * bq]);
            if (cur.sg > 0) pv += *slot;
            *slot = pv;
        }
    };

    // four steps = one turn of the register-set rotation; cur.i is the first step's tile
    auto four_steps = [&]() {
        // a run is padded to a multiple of four steps; the padding steps (wave-uniform test)
        // skip their arithmetic
        const int left = (cur.v1 - cur.v0) - cur.i;
        const float4v zero = {0.f, 0.f, 0.f, 0.f};
        float4v t0, t1 = zero, t3 = zero;
        issue_step_loads<BITS>(r3, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);
        t0 = tile_sums(r0);
        issue_step_loads<BITS>(r0, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);
        if (left > 1) t1 = tile_sums(r1);
#pragma unroll
        for (int u = 0; u < 4; ++u) t0[u] += dpp_f32<(TG == 2 ? 0x118 : 0x114)>(t1[u]);   // row_shr:8 / row_shr:4
        if (TG == 2) reduce_group(t0, cur.i);
        issue_step_loads<BITS>(r1, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);
        t1 = zero;
        if (left > 2) t1 = tile_sums(r2);
        issue_step_loads<BITS>(r2, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);
        if (left > 3) t3 = tile_sums(r3);
        if (TG == 2) {
            if (left > 2) {
#pragma unroll
                for (int u = 0; u < 4; ++u) t1[u] += dpp_f32<0x118>(t3[u]);
                reduce_group(t1, cur.i + 2);
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                t1[u] += dpp_f32<0x114>(t3[u]);
                t0[u] += dpp_f32<0x118>(t1[u]);
            }
            reduce_group(t0, cur.i);
        }
        cur.i += 4;
    };

    bool first_visit = true;
    while (!cur.done) {
        // ---- visit prologue (the barrier that ended the previous visit protects the LDS reuse)
        if (first_visit) {
#pragma unroll
            for (int u = 0; u < CFR; ++u) {
                const int e = u * NT + (int)threadIdx.x;
                if (e < nf4_first) reinterpret_cast<uint4v *>(cf_lds)[e] = cfv[u];
            }
            // the remaining two sets of the pipeline
            issue_step_loads<BITS>(r1, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);
            issue_step_loads<BITS>(r2, pf, rs_packed, kc, wave, lane); cursor_advance(pf, nseg);
            first_visit = false;
        } else {
            const int nf4 = (cur.v1 - cur.v0) * 4 * NC;   // float4 count of the visit's multipliers
            for (int e = threadIdx.x; e < nf4; e += NT)
                reinterpret_cast<uint4v *>(cf_lds)[e] = __builtin_amdgcn_raw_buffer_load_b128(rs_lut, ((uint32_t)cur.v0 * 4 * NC + e) * 16, 0, 0);
        }
        LCD_STAMP(2);
        __syncthreads();
        LCD_STAMP(3);
#pragma unroll
        for (int b = 0; b < 16; ++b) B1[b] = ((b & 3) == j) ? (_Float16)1.0f : (_Float16)0.0f;
        for (cur.sg = 0; cur.sg < nseg; ++cur.sg) {
            {   // smooth this thread's 8 activations of the segment (loaded one segment ago)
                const int g = cur.sg * NT + (int)threadIdx.x;
                half8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    o[e] = g < groups ? smooth_one((uint16_t)(xv[e >> 1] >> (16 * (e & 1))), e < 4 ? s0[e] : s1[e - 4]) : (_Float16)0.0f;
                *reinterpret_cast<half8 *>(&xs_lds[8 * threadIdx.x]) = o;
                // next segment's activations: of this visit, or segment 0 again for the next visit
                const bool more = cur.sg + 1 < nseg;
                load_x(more ? cur.sg + 1 : 0, more || cur.v1 < cur.range_end);
            }
#pragma unroll
            for (int ch = 0; ch < kBCH; ++ch)
#pragma unroll
                for (int g = 0; g < 8; ++g)   // written by this wave only: no barrier
                    A[ch][g] = *reinterpret_cast<const uint4v *>(&xs_lds[(wave * kBCH + ch) * kTileCols + 64 * q + 8 * g]);
            for (cur.i = 0; cur.i < cur.steps;) four_steps();
        }
        LCD_STAMP(4);
#ifdef LCD_TRACE
        if (lane == 0 && batch.trace && wave < 8) batch.trace[blockIdx.x * 16 + 8 + wave] = __builtin_amdgcn_s_memrealtime();
#endif
        __syncthreads();
        LCD_STAMP(5);
        // ---- visit epilogue: add the waves' slots in a fixed order, round once, store
        for (int e = threadIdx.x; e < (cur.v1 - cur.v0) * 16; e += NT) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < kBW; ++w) sum += part[w * (kVisitTiles * 16) + e];
            pb.y[(size_t)cur.v0 * kTileRows + e] = __builtin_bit_cast(uint16_t, (_Float16)sum);
        }
        cursor_next_visit(cur);
        LCD_STAMP(6);
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

    const int lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keeps addresses scalar
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

#ifdef LCD_TRACE
unsigned long long *g_trace = nullptr;
extern "C" void lcd_debug_set_trace(unsigned long long *p) { g_trace = p; }
#endif
static int g_num_cus = 0;
static int num_cus()
{
    if (g_num_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        g_num_cus = n;
    }
    return g_num_cus;
}

// One launch for a group of single-token problems.
int launch_bucket_group(const GroupItem *items, int count, int bits, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    BucketBatch batch{};
    long long cost[kMaxGroup], total = 0;
    int tiles = 0;
    for (int i = 0; i < count; ++i) {
        BucketProblem &p = batch.p[i];
        p.packed = (const uint8_t *)items[i].packed;
        p.lutA = (const float *)items[i].lut;
        p.x = items[i].x; p.s = items[i].s; p.y = items[i].y;
        p.nt = items[i].N / kTileRows; p.kc = items[i].K / kTileCols;
        cost[i] = (long long)p.nt * ((p.kc + kBSeg - 1) / kBSeg);   // steps: every row tile takes one step per segment
        total += cost[i];
        tiles += p.nt;
    }
    // Workgroups per layer.  A layer's time is that of its slowest workgroup, in units of steps:
    // a fixed start-up, then for each K segment one step per row tile plus the cost of switching
    // to the segment's activations.  A 2-bit step moves half the bytes and has no sign-flip
    // arithmetic, so the fixed costs are worth more of them.  Start from 7/8 of the proportional
    // share, then hand out the rest one by one to the layer that is slowest at that moment.
    int grid = num_cus();
    if (grid > tiles) grid = tiles;
    if (grid < count) grid = count;
    const double startup_steps = bits == 2 ? 4.0 : 2.0, segment_steps = bits == 2 ? 0.8 : 0.4;
    auto layer_time = [&](int i, int n) {
        const int segs = (batch.p[i].kc + kBSeg - 1) / kBSeg;
        const int t = (batch.p[i].nt + n - 1) / n, visits = (t + kVisitTiles - 1) / kVisitTiles;
        return startup_steps + segs * (t + visits * segment_steps);
    };
    int nwg[kMaxGroup], used = 0;
    for (int i = 0; i < count; ++i) {
        long long n = cost[i] * grid * 7 / (total * 8);
        if (n < 1) n = 1;
        if (n > batch.p[i].nt) n = batch.p[i].nt;
        nwg[i] = (int)n;
        used += nwg[i];
    }
    while (used < grid) {
        int best = -1;
        double best_time = 0.0;
        for (int i = 0; i < count; ++i) {
            if (nwg[i] >= batch.p[i].nt) continue;
            const double t = layer_time(i, nwg[i]);
            if (t > best_time) { best_time = t; best = i; }
        }
        if (best < 0) break;
        ++nwg[best];
        ++used;
    }
    grid = used;
    int acc = 0;
    for (int i = 0; i < count; ++i) {
        batch.wg_begin[i] = acc;
        acc += nwg[i];
        batch.p[i].tiles_base = batch.p[i].nt / nwg[i];
        batch.p[i].tiles_extra = batch.p[i].nt % nwg[i];
    }
    for (int i = count; i <= kMaxGroup; ++i) batch.wg_begin[i] = acc;
    batch.count = count;
#ifdef LCD_TRACE
    batch.trace = g_trace;
#endif
    const int NC = bits == 2 ? 4 : 8;
    const size_t lds = (size_t)kBSeg * kTileCols * 2 + (size_t)kVisitTiles * 16 * NC * 4 + (size_t)kBW * kVisitTiles * 16 * 4;
    static size_t lds_set[2] = {0, 0};
    const void *fn = bits == 2 ? (const void *)gemv_bucket_kernel<2> : (const void *)gemv_bucket_kernel<3>;
    if (lds > lds_set[bits - 2]) {
        if (hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)) return (int)e;
        lds_set[bits - 2] = lds;
    }
    if (bits == 2) hipLaunchKernelGGL(gemv_bucket_kernel<2>, dim3(grid), dim3(kBW * 64), lds, stream, batch);
    else hipLaunchKernelGGL(gemv_bucket_kernel<3>, dim3(grid), dim3(kBW * 64), lds, stream, batch);
    return (int)hipGetLastError();
}

int launch_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, void *workspace, const GemvPlan &plan, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    float *partial = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) + plan.xs_bytes);
    if (M == 1) {
        GroupItem it{packed, lut, x, s, y, N, K};
        return launch_bucket_group(&it, 1, bits, stream_);
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
