// Prefill path (M >= 64; any M >= 1 accepted) of the smoothed table-lookup product, gfx950.
//
// This path is a dense contraction, so it runs on v_mfma_f32_32x32x16_f16 with fp32
// accumulators (the 32x32 shape reaches the matrix peak from a single wave per SIMD; the 16x16
// shape does not).  Output tile per workgroup: 256 rows x 128 tokens, 8 waves: wave w owns rows
// [64*(w%4), +64) as two 32-row pairs, all 128 tokens as four 32-token blocks (8 accumulators of
// 16 registers, held in fixed accumulation registers) and the half w/4 of every 256-column
// chunk; the two waves of a row group add their accumulators through LDS at the end.  Two
// waves per SIMD keep the vector pipe (the dequantiser) near its full issue rate, which a single
// wave cannot reach.
//   * A operand = weights.  Lane L of the matrix instruction supplies row L%32 and 8 of the
//     step's 16 columns; it loads its own 16 bytes of the packed layout (row tile = pair's first
//     tile + (L>>4)&1) and dequantises them in registers (v_perm_b32 through the row's
//     byte-split codebook), so weights never pass through LDS.
//   * B operand = smoothed activations xs = x * rcp(s) (fp16), prepared once per call by a small
//     kernel in MFMA-operand order, so that the slice one workgroup needs per 256-column chunk
//     is one contiguous 64 KiB block.  It is copied global -> LDS with direct-to-LDS loads,
//     double buffered; every wave reads its B operands from LDS (16 bytes per lane,
//     conflict-free) through a 4-register rotating window.
// Each decoded A operand is used for 4 token blocks, each B operand for 2 row pairs.
#include <hip/hip_runtime.h>
#include <algorithm>
#include "lcd_internal.h"
#include "lcd_device.h"
#include "lcd_launch.h"

namespace lcd {

// packed weights are read by every token block of the layer: default cache policy (the non-temporal
// hint of the decode kernels costs 2 % here)
constexpr int kGemmWeightPolicy = 0;
constexpr int kXcds = 8;             // accelerator complex dies of the MI355X, each with its own L2
constexpr int kGemmRowGroups = 4;   // 64-row groups per workgroup
constexpr int kGemmWaves = 2 * kGemmRowGroups;   // x the two halves of a chunk
constexpr int kGemmPairs = 2;        // 32-row pairs per wave
constexpr int kGemmTokBlks = 4;      // 32-token blocks per workgroup (shared by its waves)
constexpr int kGemmTokens = 32 * kGemmTokBlks;
constexpr int kStageBytes = kGemmTokBlks * 16 * 1024;  // 64 KiB: 4 token blocks x 16 k-steps x 1 KiB

typedef __attribute__((address_space(3))) uint32_t lds_u32;
typedef __attribute__((address_space(1))) const uint32_t glb_u32;

// ---- accumulators in fixed accumulation registers ------------------------------------------------
// The 8 accumulators of a wave (16 registers each) live in a[0:127] and are touched only by the
// inline assembly below, so the compiler never copies them (as loop-carried values it would move
// all 128 registers to VGPRs and back in every iteration).  This file is compiled with AGPR
// spilling disabled, and uses no MFMA builtins, so the compiler itself never allocates an AGPR.
// The compiler does not look inside the assembly text, so it cannot keep the distance the hardware
// requires between a vector instruction that writes a register and a matrix instruction that reads it
// as an operand (it is free to place the last instruction of an operand's dequantisation directly in
// front of the matrix instruction, and does so depending on unrelated details of the source): every
// matrix instruction therefore brings its own two wait states.  Two waves share a SIMD and a 32x32x16
// instruction occupies the matrix pipe for 32 cycles, so the two issue cycles are hidden.
template <int IDX> __device__ __forceinline__ void mfma_acc(uint4v a, uint4v b);
template <int IDX> __device__ __forceinline__ float16v read_acc();
template <int IDX> __device__ __forceinline__ void zero_acc();
// Register names cannot be computed inside assembly text, so each accumulator lists its 16 registers once.
#define LCD_ACC_CLOBBERS(r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11, r12, r13, r14, r15)                                   \
    "a" #r0, "a" #r1, "a" #r2, "a" #r3, "a" #r4, "a" #r5, "a" #r6, "a" #r7, "a" #r8, "a" #r9, "a" #r10, "a" #r11, "a" #r12,      \
        "a" #r13, "a" #r14, "a" #r15
#define LCD_ACC_READ(n, r) "v_accvgpr_read_b32 %" #n ", a" #r
#define LCD_ACC_ZERO(r) "v_accvgpr_write_b32 a" #r ", 0"
#define LCD_ACCUMULATOR(IDX, r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11, r12, r13, r14, r15)                                \
    template <> __device__ __forceinline__ void mfma_acc<IDX>(uint4v a, uint4v b)                                                 \
    {                                                                                                                              \
        asm volatile("s_nop 1\n\tv_mfma_f32_32x32x16_f16 a[" #r0 ":" #r15 "], %0, %1, a[" #r0 ":" #r15 "]"                     \
                     :                                                                                                             \
                     : "v"(a), "v"(b)                                                                                              \
                     : LCD_ACC_CLOBBERS(r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11, r12, r13, r14, r15));                    \
    }                                                                                                                              \
    template <> __device__ __forceinline__ float16v read_acc<IDX>()                                                                \
    {                                                                                                                              \
        float t[16];                                                                                                               \
        asm volatile(LCD_ACC_READ(0, r0) "\n\t" LCD_ACC_READ(1, r1) "\n\t" LCD_ACC_READ(2, r2) "\n\t" LCD_ACC_READ(3, r3) "\n\t"   \
                     LCD_ACC_READ(4, r4) "\n\t" LCD_ACC_READ(5, r5) "\n\t" LCD_ACC_READ(6, r6) "\n\t" LCD_ACC_READ(7, r7) "\n\t"   \
                     LCD_ACC_READ(8, r8) "\n\t" LCD_ACC_READ(9, r9) "\n\t" LCD_ACC_READ(10, r10) "\n\t" LCD_ACC_READ(11, r11)      \
                     "\n\t" LCD_ACC_READ(12, r12) "\n\t" LCD_ACC_READ(13, r13) "\n\t" LCD_ACC_READ(14, r14) "\n\t"                 \
                     LCD_ACC_READ(15, r15)                                                                                         \
                     : "=v"(t[0]), "=v"(t[1]), "=v"(t[2]), "=v"(t[3]), "=v"(t[4]), "=v"(t[5]), "=v"(t[6]), "=v"(t[7]),             \
                       "=v"(t[8]), "=v"(t[9]), "=v"(t[10]), "=v"(t[11]), "=v"(t[12]), "=v"(t[13]), "=v"(t[14]), "=v"(t[15]));      \
        float16v v;                                                                                                                \
        for (int i = 0; i < 16; ++i) v[i] = t[i];                                                                                  \
        return v;                                                                                                                  \
    }                                                                                                                              \
    template <> __device__ __forceinline__ void zero_acc<IDX>()                                                                    \
    {                                                                                                                              \
        asm volatile(LCD_ACC_ZERO(r0) "\n\t" LCD_ACC_ZERO(r1) "\n\t" LCD_ACC_ZERO(r2) "\n\t" LCD_ACC_ZERO(r3) "\n\t"               \
                     LCD_ACC_ZERO(r4) "\n\t" LCD_ACC_ZERO(r5) "\n\t" LCD_ACC_ZERO(r6) "\n\t" LCD_ACC_ZERO(r7) "\n\t"               \
                     LCD_ACC_ZERO(r8) "\n\t" LCD_ACC_ZERO(r9) "\n\t" LCD_ACC_ZERO(r10) "\n\t" LCD_ACC_ZERO(r11) "\n\t"             \
                     LCD_ACC_ZERO(r12) "\n\t" LCD_ACC_ZERO(r13) "\n\t" LCD_ACC_ZERO(r14) "\n\t" LCD_ACC_ZERO(r15)                  \
                     :                                                                                                             \
                     :                                                                                                             \
                     : LCD_ACC_CLOBBERS(r0, r1, r2, r3, r4, r5, r6, r7, r8, r9, r10, r11, r12, r13, r14, r15));                    \
    }
LCD_ACCUMULATOR(0, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15)
LCD_ACCUMULATOR(1, 16, 17, 18, 19, 20, 21, 22, 23, 24, 25, 26, 27, 28, 29, 30, 31)
LCD_ACCUMULATOR(2, 32, 33, 34, 35, 36, 37, 38, 39, 40, 41, 42, 43, 44, 45, 46, 47)
LCD_ACCUMULATOR(3, 48, 49, 50, 51, 52, 53, 54, 55, 56, 57, 58, 59, 60, 61, 62, 63)
LCD_ACCUMULATOR(4, 64, 65, 66, 67, 68, 69, 70, 71, 72, 73, 74, 75, 76, 77, 78, 79)
LCD_ACCUMULATOR(5, 80, 81, 82, 83, 84, 85, 86, 87, 88, 89, 90, 91, 92, 93, 94, 95)
LCD_ACCUMULATOR(6, 96, 97, 98, 99, 100, 101, 102, 103, 104, 105, 106, 107, 108, 109, 110, 111)
LCD_ACCUMULATOR(7, 112, 113, 114, 115, 116, 117, 118, 119, 120, 121, 122, 123, 124, 125, 126, 127)
#undef LCD_ACCUMULATOR
#undef LCD_ACC_ZERO
#undef LCD_ACC_READ
#undef LCD_ACC_CLOBBERS
__device__ __forceinline__ void zero_accs()
{
    zero_acc<0>(); zero_acc<1>(); zero_acc<2>(); zero_acc<3>(); zero_acc<4>(); zero_acc<5>(); zero_acc<6>(); zero_acc<7>();
}

// One lane's packed words of a chunk half: per pair, the lane's row and the 64 columns
// [64*(2*half + L>>5), +64) of the chunk.
template <int BITS>
struct GemmTileRegs {
    uint4v lo[kGemmPairs];
    uint2v hi[kGemmPairs];    // 3 bits: the third-bit words
    uint4v hi4[kGemmPairs];   // 4 bits: the second plane
};

// byte-split codebook of a lane's row: two words of each kind up to 3 bits, four with 4 bits
template <int BITS> struct GemmTables { typedef RowTables type; };
template <> struct GemmTables<4> { typedef RowTables4 type; };

template <int BITS>
__device__ __forceinline__ void load_gemm_tiles(GemmTileRegs<BITS> &r, __amdgpu_buffer_rsrc_t packed, int t0, int nt,
                                                int kc, int c, int h, int lane)
{
    constexpr uint32_t TB = kTileRows * kTileCols * BITS / 8;
    const int sub = (lane >> 4) & 1, kh = lane >> 5, i = lane & 15;
#pragma unroll
    for (int p = 0; p < kGemmPairs; ++p) {
        const int tile = t0 + 2 * p + sub;
        const uint32_t base = ((uint32_t)tile * (uint32_t)kc + (uint32_t)c) * TB;
        const int slot = 16 * (2 * h + kh) + i;          // lane slot inside the 16 x 256 tile
        const bool v = tile < nt;
        r.lo[p] = __builtin_amdgcn_raw_buffer_load_b128(packed, v ? base + 16 * slot : 0xFFFFFFF0u, 0, kGemmWeightPolicy);
        if (BITS == 3) r.hi[p] = __builtin_amdgcn_raw_buffer_load_b64(packed, v ? base + 1024 + 8 * slot : 0xFFFFFFF0u, 0, kGemmWeightPolicy);
        if (BITS == 4) r.hi4[p] = __builtin_amdgcn_raw_buffer_load_b128(packed, v ? base + 1024 + 16 * slot : 0xFFFFFFF0u, 0, kGemmWeightPolicy);
    }
}

// copy one 64 KiB stage: every wave copies 8 KiB as 8 wave-wide 1 KiB direct-to-LDS loads,
// blocks [first, first + count) of them per call (the copy is spread over a word's matrix steps)
__device__ __forceinline__ void stage_copy(const uint8_t *__restrict__ src, uint8_t *lds_dst, int wave, int lane, int first, int count)
{
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        if (u < first || u >= first + count) continue;
        const int blk = wave * 8 + u;  // 1 KiB block index inside the stage
        __builtin_amdgcn_global_load_lds((glb_u32 *)(src + (size_t)blk * 1024 + lane * 16),
                                         (lds_u32 *)(lds_dst + blk * 1024), 16, 0, 0);
    }
}

// B operands (16 bytes per lane) rotate through a window of four registers: the read for
// matrix step s+3 is issued while step s computes.  A stage holds blocks
// [token block 4][half 2][k-step 8] of 1 KiB.  The reads and the waits for them are written out
// (LDS reads of a wave return in order, so "at most n newer reads outstanding" is the exact
// condition for a window slot; left to itself the compiler waited for ALL outstanding reads at
// every fourth step, which emptied the window each time).
struct BWindow { uint4v w[4]; };

// `base` = 32-bit LDS address of (stage + half * 8 KiB + the lane's 16 bytes)
template <int G, int TBLK>
__device__ __forceinline__ uint4v read_b(uint32_t base)
{
    uint4v v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(base), "n"((TBLK * 16 + G) * 1024) : "memory");
    return v;
}
template <int N>
__device__ __forceinline__ void lds_wait()
{
    asm volatile("s_waitcnt lgkmcnt(%0)" : : "n"(N) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const uint8_t *p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint8_t *)p;
}

// The dequantiser's first two stages for quarter T of word DN of pair P, for any width: the selector
// (4 bits: and the pool word), then the table lookups.
template <int BITS, int DN, int T>
__device__ __forceinline__ void gemm_select(const GemmTileRegs<BITS> &r, int p, const HighBits &hb, uint32_t &sel, uint32_t &pool)
{
    if constexpr (BITS == 4) decode_select4<T>(r.lo[p][DN], r.hi4[p][DN], sel, pool);
    else sel = decode_select<BITS, DN, T>(r.lo[p][DN], hb);
}
template <int BITS>
__device__ __forceinline__ void gemm_lookup(uint32_t sel, uint32_t pool, const typename GemmTables<BITS>::type &tb, uint32_t &lo, uint32_t &hi)
{
    if constexpr (BITS == 4) decode_lookup4(sel, pool, tb, lo, hi);
    else decode_lookup<BITS>(sel, tb, lo, hi);
}

// Decoded A operands of one packed word: [pair][k-step of the word].
struct WordOps { uint4v op[kGemmPairs][2]; };

// One packed word per pair (16 weights per lane) = two k-steps x 4 token blocks = 8 matrix steps
// of 2 MFMAs.  The word's operands `cur` were decoded during the previous word; each matrix step
// also decodes one eighth of the NEXT word (word DN of `rn`) into `nxt`, so that vector and
// matrix instructions alternate in every wave's stream instead of coming in bursts (two waves of
// a SIMD leave a barrier in phase; with bursts both would decode, then both would multiply).
// COPY: the step also issues its share of the next stage's global -> LDS copy.
// On entry the B window holds steps 0..2 of this word; on exit steps 0..2 of the next word of the
// chunk (the caller primes it again after the last word).
template <int BITS, int D, int DN, bool COPY>
__device__ __forceinline__ void gemm_word(const WordOps &cur, WordOps &nxt, const GemmTileRegs<BITS> &rn,
                                          const HighBits (&hbn)[kGemmPairs], const typename GemmTables<BITS>::type (&tb)[kGemmPairs],
                                          uint32_t bbase, BWindow &bw,
                                          const uint8_t *copy_src, uint8_t *copy_dst, int wave, int lane)
{
#define LCD_GEMM_FENCE __builtin_amdgcn_sched_barrier(0);
    uint32_t sel = 0, pool = 0;
#define LCD_GEMM_STEP(ST)                                                                                   \
    {                                                                                                       \
        constexpr int st = ST, a = st >> 2, blk = st & 3, nx = st + 3, np = st >> 2, nt4 = st & 3;          \
        uint32_t lo, hi, o0, o1;                                                                            \
        /* prefetch step st+3 into the slot that step st-1 used */                                          \
        if (nx < 8) bw.w[nx & 3] = read_b<2 * D + (nx >> 2), (nx & 3)>(bbase);                              \
        else if (D < 3) bw.w[nx & 3] = read_b<(2 * D + 2) & 7, (nx - 8) & 3>(bbase);                        \
        if (st == 0) gemm_select<BITS, DN, 0>(rn, 0, hbn[0], sel, pool);                                    \
        /* reads newer than this step's operand: 3, fewer at the end of a chunk's last word */             \
        lds_wait<(D < 3 || st <= 4) ? 3 : 7 - st>();                                                        \
        mfma_acc<blk>(cur.op[0][a], bw.w[st & 3]);                                                          \
        /* the vector work of the step is split behind the two matrix instructions: the second one     */ \
        /* cannot issue before the first has left the pipe, and a wave issues in order.  Lookups of     */ \
        /* quarter st, then the selector of quarter st+1, then the interleave: dependent instructions   */ \
        /* stay a few issue slots apart.                                                                 */ \
        if (COPY && copy_src) stage_copy(copy_src, copy_dst, wave, lane, st, 1);                            \
        gemm_lookup<BITS>(sel, pool, tb[np], lo, hi);                                                       \
        LCD_GEMM_FENCE                                                                                      \
        mfma_acc<4 + blk>(cur.op[1][a], bw.w[st & 3]);                                                      \
        if (st < 7) gemm_select<BITS, DN, (st + 1) & 3>(rn, (st + 1) >> 2, hbn[(st + 1) >> 2], sel, pool);  \
        decode_interleave(lo, hi, o0, o1);                                                                  \
        nxt.op[np][0][nt4] = o0; nxt.op[np][1][nt4] = o1;                                                   \
        LCD_GEMM_FENCE                                                                                      \
    }
    LCD_GEMM_STEP(0) LCD_GEMM_STEP(1) LCD_GEMM_STEP(2) LCD_GEMM_STEP(3)
    LCD_GEMM_STEP(4) LCD_GEMM_STEP(5) LCD_GEMM_STEP(6) LCD_GEMM_STEP(7)
#undef LCD_GEMM_STEP
}


// One output tile (row block bx, token block by) of one layer: the whole life of a workgroup.
template <int BITS>
__device__ __forceinline__ void gemm_tile(const uint8_t *__restrict__ packed_, const uint8_t *__restrict__ lutB, const uint8_t *__restrict__ xs,
                                          uint16_t *__restrict__ y, int M, int Mpad, int N, int K, int bx, int by, uint8_t *lds,
                                          float out_scale)   // 1, or the quantisation step when xs holds INT8 codes (Eq. 11)
{
    constexpr uint32_t TB = kTileRows * kTileCols * BITS / 8;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keeps addresses scalar
    const int kc = K / kTileCols, nt = N / kTileRows;
    const int rgrp = wave & (kGemmRowGroups - 1), khalf = wave >> 2;     // row group and chunk half of this wave
    const int t0 = (bx * kGemmRowGroups + rgrp) * (2 * kGemmPairs);      // first row tile of this wave
    const int tb0 = by * kGemmTokBlks;                                   // first 32-token block of this workgroup
    const int boff = lane * 16;                                           // lane's 16 bytes inside a 1 KiB operand block
    const __amdgpu_buffer_rsrc_t packed = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(packed_), 0, (uint32_t)nt * (uint32_t)kc * TB, 0x00020000);

    // activations of chunk c for this workgroup's 128 tokens: one contiguous 64 KiB block
    const size_t chunk_stride = (size_t)(Mpad >> 5) * 16 * 1024;
    const uint8_t *xs_base = xs + (size_t)tb0 * 16 * 1024;

    // this lane's row in each pair, and its byte-split codebook
    typename GemmTables<BITS>::type tb[kGemmPairs];
#pragma unroll
    for (int p = 0; p < kGemmPairs; ++p) {
        const int tile = min(t0 + 2 * p + ((lane >> 4) & 1), nt - 1);
        const int row = tile * kTileRows + (lane & 15);
        if constexpr (BITS == 2) {
            const uint2v v = *reinterpret_cast<const uint2v *>(lutB + (size_t)row * 8);
            tb[p].lo[0] = v[0]; tb[p].hi[0] = v[1]; tb[p].lo[1] = 0; tb[p].hi[1] = 0;
        } else if constexpr (BITS == 3) {
            const uint4v v = *reinterpret_cast<const uint4v *>(lutB + (size_t)row * 16);
            tb[p].lo[0] = v[0]; tb[p].lo[1] = v[1]; tb[p].hi[0] = v[2]; tb[p].hi[1] = v[3];
        } else {
            const uint4v v = *reinterpret_cast<const uint4v *>(lutB + (size_t)row * 32);
            const uint4v w = *reinterpret_cast<const uint4v *>(lutB + (size_t)row * 32 + 16);
#pragma unroll
            for (int u = 0; u < 4; ++u) { tb[p].lo[u] = v[u]; tb[p].hi[u] = w[u]; }
        }
    }
    zero_accs();

    GemmTileRegs<BITS> r0, r1;
    load_gemm_tiles<BITS>(r0, packed, t0, nt, kc, 0, khalf, lane);
    stage_copy(xs_base, lds, wave, lane, 0, 8);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    auto high_bits = [&](const GemmTileRegs<BITS> &r, HighBits (&hb)[kGemmPairs]) {
#pragma unroll
        for (int p = 0; p < kGemmPairs; ++p) {
            hb[p] = HighBits{0u, 0u};
            if (BITS == 3) hb[p] = regroup_high(r.hi[p]);
        }
    };

    BWindow bw;
    WordOps wa, wb;          // operands of the current / next word, swapping roles word by word
    HighBits hb[kGemmPairs], hbn[kGemmPairs];
    // Chunk c is computed from LDS stage c&1 and register set r; word D's matrix steps decode word
    // D+1, the last word's decode the first word of chunk c+1 (set rn, loaded at the top of chunk
    // c).  The copy of chunk c+1's stage is issued during word 0 (the other stage was released by
    // the barrier that ended chunk c-1) and has the whole chunk to land: one wait + one barrier
    // per chunk, after which the B window is primed from the new stage.
    auto compute = [&](const GemmTileRegs<BITS> &r, const GemmTileRegs<BITS> &rn, const uint8_t *stage,
                       uint8_t *other_stage, const uint8_t *copy_src) {
        const uint32_t bbase = lds_address(stage) + khalf * 8 * 1024 + boff;
        const uint32_t obase = lds_address(other_stage) + khalf * 8 * 1024 + boff;
        gemm_word<BITS, 0, 1, true>(wa, wb, r, hb, tb, bbase, bw, copy_src, other_stage, wave, lane);
        gemm_word<BITS, 1, 2, false>(wb, wa, r, hb, tb, bbase, bw, nullptr, nullptr, wave, lane);
        gemm_word<BITS, 2, 3, false>(wa, wb, r, hb, tb, bbase, bw, nullptr, nullptr, wave, lane);
        high_bits(rn, hbn);
        gemm_word<BITS, 3, 0, false>(wb, wa, rn, hbn, tb, bbase, bw, nullptr, nullptr, wave, lane);
#pragma unroll
        for (int p = 0; p < kGemmPairs; ++p) hb[p] = hbn[p];
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();   // the next stage has landed for every wave, and every wave is done with this one
        bw.w[0] = read_b<0, 0>(obase);
        bw.w[1] = read_b<0, 1>(obase);
        bw.w[2] = read_b<0, 2>(obase);
    };

    // prologue: B operands of the first three steps, operands of the first word
    {
        const uint32_t base0 = lds_address(lds) + khalf * 8 * 1024 + boff;
        bw.w[0] = read_b<0, 0>(base0);
        bw.w[1] = read_b<0, 1>(base0);
        bw.w[2] = read_b<0, 2>(base0);
    }
    high_bits(r0, hb);
#pragma unroll
    for (int p = 0; p < kGemmPairs; ++p) {
        if constexpr (BITS == 4) decode_word4(r0.lo[p][0], r0.hi4[p][0], tb[p], wa.op[p][0], wa.op[p][1]);
        else decode_word<BITS, 0>(r0.lo[p][0], hb[p], tb[p], wa.op[p][0], wa.op[p][1]);
    }
    for (int c = 0; c < kc; c += 2) {
        // even chunk: compute from stage 0 / r0 while chunk c+1 lands in stage 1 / r1
        const bool more1 = c + 1 < kc;
        if (more1) load_gemm_tiles<BITS>(r1, packed, t0, nt, kc, c + 1, khalf, lane);
        compute(r0, r1, lds, lds + kStageBytes, more1 ? xs_base + (size_t)(c + 1) * chunk_stride : nullptr);
        if (!more1) break;
        const bool more2 = c + 2 < kc;
        if (more2) load_gemm_tiles<BITS>(r0, packed, t0, nt, kc, c + 2, khalf, lane);
        compute(r1, r0, lds + kStageBytes, lds, more2 ? xs_base + (size_t)(c + 2) * chunk_stride : nullptr);
    }

    // The two waves of a row group hold partial sums over the two halves of every chunk.  Each keeps
    // one 32-row pair and hands the other pair's four accumulators to its partner through LDS (the
    // stages are free now): per row group two 16 KiB areas, area h read by the wave with khalf == h,
    // [accumulator 4][register quad 4][lane] float4.
    // The accumulator reads below are assembly text too: the distance the hardware requires between a
    // matrix instruction's register write and a vector instruction's read of it (19 wait states for
    // the 16-pass instruction) is kept here by hand, once per workgroup.
    asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
    float4v *area_in = reinterpret_cast<float4v *>(lds) + (size_t)(rgrp * 2 + khalf) * (4 * 4 * 64);
    float4v *area_out = reinterpret_cast<float4v *>(lds) + (size_t)(rgrp * 2 + (khalf ^ 1)) * (4 * 4 * 64);
    auto put_acc = [&](const float16v &v, int slot) {
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) area_out[(slot * 4 + rg) * 64 + lane] = float4v{v[4 * rg], v[4 * rg + 1], v[4 * rg + 2], v[4 * rg + 3]};
    };
    if (khalf == 0) { put_acc(read_acc<4>(), 0); put_acc(read_acc<5>(), 1); put_acc(read_acc<6>(), 2); put_acc(read_acc<7>(), 3); }
    else            { put_acc(read_acc<0>(), 0); put_acc(read_acc<1>(), 1); put_acc(read_acc<2>(), 2); put_acc(read_acc<3>(), 3); }
    __syncthreads();

    // Sum of the two halves, rounded once to fp16.  Accumulator register r of lane l is row
    // 8*(r/4) + 4*(l/32) + r%4 of the pair, token l%32: four consecutive rows of one token per
    // register quad, i.e. 8-byte pieces of 32 different output rows per store instruction.  Stored
    // like that, every 128-byte line of y is written in 16 pieces and the end of the kernel waits
    // on the L2's request rate; so the wave first turns its 32 rows x 128 tokens into
    // [token][row] order through the area it has just read (nobody else touches it any more) and
    // then writes 64 contiguous bytes per token: 4 lanes x 16 bytes, the other half of the line
    // coming from its partner.
    const int tok = lane & 31, lh = lane >> 5;
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    constexpr int kOutStride = 32 * 2 + 16;   // bytes per token row of the tile (16-byte aligned, spreads the banks)
    uint8_t *tile_out = reinterpret_cast<uint8_t *>(area_in);
    uint2v outv[4][4];
    auto sum_acc = [&](const float16v &own, int slot) {
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const float4v other = area_in[(slot * 4 + rg) * 64 + lane];
            half4 o;
#pragma unroll
            for (int u = 0; u < 4; ++u) o[u] = (_Float16)((own[4 * rg + u] + other[u]) * out_scale);
            outv[slot][rg] = __builtin_bit_cast(uint2v, o);
        }
    };
    if (khalf == 0) { sum_acc(read_acc<0>(), 0); sum_acc(read_acc<1>(), 1); sum_acc(read_acc<2>(), 2); sum_acc(read_acc<3>(), 3); }
    else            { sum_acc(read_acc<4>(), 0); sum_acc(read_acc<5>(), 1); sum_acc(read_acc<6>(), 2); sum_acc(read_acc<7>(), 3); }
    // every read above must precede the writes below, which reuse the same bytes: the wait orders
    // them for the compiler too (the two sides use different vector types)
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
#pragma unroll
        for (int rg = 0; rg < 4; ++rg)
            *reinterpret_cast<uint2v *>(tile_out + (blk * 32 + tok) * kOutStride + (8 * rg + 4 * lh) * 2) = outv[blk][rg];
    }
    asm volatile("" ::: "memory");               // LDS operations of one wave complete in order; keep the compiler's order too
    const int r4 = lane & 3;                       // which 8 rows of the pair's 32
    const int tile_first = t0 + 2 * khalf;         // first 16-row tile of this wave's pair
    const bool rows_ok = tile_first + (r4 >> 1) < nt;   // N is a multiple of 16: 8 rows are all inside or all outside
#pragma unroll
    for (int it = 0; it < kGemmTokens / 16; ++it) {
        const int tk = it * 16 + (lane >> 2);
        const uint4v v = *reinterpret_cast<const uint4v *>(tile_out + tk * kOutStride + r4 * 16);
        const int m = tb0 * 32 + tk;
        if (m < M && rows_ok) *reinterpret_cast<uint4v *>(y + (size_t)m * N + (size_t)tile_first * kTileRows + r4 * 8) = v;
    }
}

// XCD-aware tile order.  Workgroup ids go round-robin over the 8 XCDs, each with its own L2.
// Output tiles are numbered token-block-major and cut into 8 contiguous runs, one per XCD, so
// the workgroups that are resident on an XCD at the same time share one or two 128-token
// blocks of activations (1 MiB each at K = 4096), which then stay in that XCD's 4 MiB L2.
template <int BITS>
__global__ void __launch_bounds__(kGemmWaves * 64, 1)
gemm_kernel(const uint8_t *__restrict__ packed_, const uint8_t *__restrict__ lutB, const uint8_t *__restrict__ xs,
            uint16_t *__restrict__ y, int M, int Mpad, int N, int K, int grid_rows, int tiles_per_xcd, float out_scale)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];  // 2 stages x 64 KiB
    const int out_tile = (int)(blockIdx.x % kXcds) * tiles_per_xcd + (int)(blockIdx.x / kXcds);
    const int total_tiles = grid_rows * (Mpad / kGemmTokens);
    if ((int)(blockIdx.x / kXcds) >= tiles_per_xcd || out_tile >= total_tiles) return;
    gemm_tile<BITS>(packed_, lutB, xs, y, M, Mpad, N, K, out_tile % grid_rows, out_tile / grid_rows, lds, out_scale);
}

// Several layers in one launch (same token count and index width): every XCD's queue of
// workgroups holds its run of every layer's tiles, layer after layer in the order of the batch
// (the host puts the layers with the longest tiles first), so the tail of one layer is filled by
// the head of the next and only the last layer leaves compute units idle at the end.
struct GemmProblem {
    const uint8_t *packed, *lutB, *xs;
    uint16_t *y;
    int N, K, grid_rows, tiles_per_xcd;
    int queue_begin;   // position of this layer's first tile in an XCD's queue
    float out_scale;   // 1, or the layer's activation quantisation step
};
struct GemmBatch {
    GemmProblem p[kMaxGroup];
    int count, M, Mpad;
};
template <int BITS>
__global__ void __launch_bounds__(kGemmWaves * 64, 1) gemm_group_kernel(const GemmBatch batch)
{
    extern __shared__ __attribute__((aligned(1024))) uint8_t lds[];  // 2 stages x 64 KiB
    const int xcd = (int)(blockIdx.x % kXcds), pos = (int)(blockIdx.x / kXcds);
    int pi = 0;
    for (int i = 1; i < batch.count; ++i) pi += pos >= batch.p[i].queue_begin ? 1 : 0;   // queue_begin grows with i
    const GemmProblem pb = batch.p[pi];
    const int out_tile = xcd * pb.tiles_per_xcd + (pos - pb.queue_begin);
    if (out_tile >= pb.grid_rows * (batch.Mpad / kGemmTokens)) return;
    gemm_tile<BITS>(pb.packed, pb.lutB, pb.xs, pb.y, batch.M, batch.Mpad, pb.N, pb.K, out_tile % pb.grid_rows, out_tile / pb.grid_rows, lds,
                    pb.out_scale);
}

int launch_gemm(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, float act_scale, void *workspace, const GemmPlan &plan, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    const int Mpad = plan.m_pad;
    if (int e = launch_smooth(x, s, workspace, M, Mpad, K, act_scale, stream)) return e;
    // byte-split tables: behind the bucket multipliers (2 and 3 bits), the whole table (4 bits)
    const uint8_t *lutB = static_cast<const uint8_t *>(lut) + (bits == 4 ? 0 : (size_t)N * (bits == 2 ? 4 : 8) * 4);
    const int nt = N / kTileRows;
    const int tiles_per_wg = kGemmRowGroups * 2 * kGemmPairs;
    const int grid_rows = (nt + tiles_per_wg - 1) / tiles_per_wg;
    const int total_tiles = grid_rows * (Mpad / kGemmTokens);
    const int tiles_per_xcd = (total_tiles + kXcds - 1) / kXcds;
    const dim3 grid(tiles_per_xcd * kXcds), block(kGemmWaves * 64);
    const size_t lds_bytes = 2 * kStageBytes;
    static PerDeviceFlags<3> lds_raised;
    const void *fn = bits == 2 ? (const void *)gemm_kernel<2> : bits == 3 ? (const void *)gemm_kernel<3> : (const void *)gemm_kernel<4>;
    if (hipError_t e = raise_lds_limit_once(lds_raised, bits - 2, fn, lds_bytes)) return (int)e;
    const uint8_t *packed_arg = static_cast<const uint8_t *>(packed), *xs_arg = static_cast<const uint8_t *>(workspace);
    int M_arg = M, Mpad_arg = Mpad, N_arg = N, K_arg = K, rows_arg = grid_rows, xcd_arg = tiles_per_xcd;
    float scale_arg = act_scale != 0.0f ? act_scale : 1.0f;
    void *args[] = {&packed_arg, &lutB, &xs_arg, &y, &M_arg, &Mpad_arg, &N_arg, &K_arg, &rows_arg, &xcd_arg, &scale_arg};
    if (hipError_t e = hipLaunchKernel(fn, grid, block, args, lds_bytes, stream)) return (int)e;
    return (int)hipGetLastError();
}

int launch_gemm_group(const GroupItem *items, int count, int M, int bits, void *workspace, void *stream_)
{
    hipStream_t stream = (hipStream_t)stream_;
    const int Mpad = plan_gemm(M, items[0].N, items[0].K, bits).m_pad;
    // layers with the longest tiles (largest K) first in every XCD's queue
    int order[kMaxGroup];
    for (int i = 0; i < count; ++i) order[i] = i;
    std::stable_sort(order, order + count, [&](int a, int b) { return items[a].K > items[b].K; });
    // Layers that read the same input (same x, s, K and quantisation step: q/k/v, gate/up of a decoder
    // block) share one transformed copy of it: the activations are smoothed once per distinct input.
    SmoothItem sm[kMaxGroup];
    int distinct = 0;
    GemmBatch batch{};
    size_t offset = 0;
    int queue = 0;
    for (int q = 0; q < count; ++q) {
        const GroupItem &it = items[order[q]];
        uint8_t *xs = nullptr;
        for (int d = 0; d < distinct && !xs; ++d)
            if (sm[d].x == it.x && sm[d].s == it.s && sm[d].K == it.K && sm[d].s_q == it.act_scale) xs = static_cast<uint8_t *>(sm[d].xs);
        if (!xs) {
            xs = static_cast<uint8_t *>(workspace) + offset;
            offset += plan_gemm(M, it.N, it.K, bits).xs_bytes;
            sm[distinct++] = SmoothItem{it.x, it.s, xs, it.K, it.act_scale};
        }
        GemmProblem &p = batch.p[q];
        p.packed = static_cast<const uint8_t *>(it.packed);
        p.lutB = static_cast<const uint8_t *>(it.lut) + (bits == 4 ? 0 : (size_t)it.N * (bits == 2 ? 4 : 8) * 4);
        p.xs = xs;
        p.y = it.y;
        p.N = it.N; p.K = it.K;
        const int nt = it.N / kTileRows, tiles_per_wg = kGemmRowGroups * 2 * kGemmPairs;
        p.grid_rows = (nt + tiles_per_wg - 1) / tiles_per_wg;
        const int total_tiles = p.grid_rows * (Mpad / kGemmTokens);
        p.tiles_per_xcd = (total_tiles + kXcds - 1) / kXcds;
        p.queue_begin = queue;
        p.out_scale = it.act_scale != 0.0f ? it.act_scale : 1.0f;
        queue += p.tiles_per_xcd;
    }
    batch.count = count; batch.M = M; batch.Mpad = Mpad;
    if (int e = launch_smooth_group(sm, distinct, M, Mpad, stream)) return e;
    const size_t lds_bytes = 2 * kStageBytes;
    static PerDeviceFlags<3> lds_raised;
    const void *fn = bits == 2 ? (const void *)gemm_group_kernel<2> : bits == 3 ? (const void *)gemm_group_kernel<3> : (const void *)gemm_group_kernel<4>;
    if (hipError_t e = raise_lds_limit_once(lds_raised, bits - 2, fn, lds_bytes)) return (int)e;
    void *args[] = {&batch};
    if (hipError_t e = hipLaunchKernel(fn, dim3((unsigned)queue * kXcds), dim3(kGemmWaves * 64), args, lds_bytes, stream)) return (int)e;
    return (int)hipGetLastError();
}


}  // namespace lcd
