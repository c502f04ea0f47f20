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
// The sign flips cost one xor-and (v_bitop3_b32) per pair of weights plus one 64-bit shift per
// two pairs.
// Two tokens at 2 bits take the sign-flipped pass's place with the second token's activations.
// With the INT8 activation codes of Sec. 4.1 at 2 bits, A holds the codes as int8 numbers and the
// instruction is v_smfmac_i32_16x16x128_i8 (64 values per row and instruction): one to four tokens.
//
// Work split: the 8 waves of a workgroup split K into segments of 16 chunks (256 columns each),
// two chunks per wave, and keep their chunks' activations in registers for a whole segment; the
// workgroup walks over its row tiles (16 rows) segment by segment, every wave streaming two
// KiB-sized contiguous pieces of the packed matrix per tile.  The waves' partial outputs meet in
// LDS and are added in a fixed order; K of any length stays inside one workgroup.
#include <hip/hip_runtime.h>
#include <type_traits>
#include <algorithm>
#include <mutex>
#include "lcd_internal.h"
#include "lcd_device.h"
#include "lcd_launch.h"


namespace lcd {

// Cache policy of the packed-index loads: non-temporal.  Every index byte is read exactly once per
// launch, and without the hint the stream pushes the small reused data (activations, smoothing
// factors, codebook tables) out of the caches: measured +4 % (7B set, 3 bits) to +8 % (70B MLP, 2
// bits) on the single-token kernel, +3.5 % on the tokens kernel.  (Bit 1 of the buffer
// instructions' cache-policy operand is "nt" on gfx950.)
constexpr int kStreamPolicy = 2;



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
//   segments   the 8 waves split K into segments of 16 chunks (two 256-column chunks per wave).
//              For each segment a wave smooths its own activations (x / s), fans them out to the
//              lanes through its own piece of LDS (no workgroup synchronisation) and keeps them
//              in registers, then streams the visit's row tiles: 2-3 KiB of packed indices per
//              tile, 16-32 sparse MFMAs, and (once per 2 or 4 tiles) a few VALU ops that turn
//              bucket sums into partial outputs with the per-bucket multipliers (prefetched from
//              the table together with the tiles), which the wave adds into its own LDS slot;
//   epilogue   one barrier; the workgroup adds the 8 waves' slots in a fixed order, stores y.
// Loads of packed indices run kSets-1 steps ahead of the arithmetic, across segment and visit
// boundaries.  Matrix and vector instructions of one SIMD do not overlap in time (measured), so
// the instruction count per byte is what matters, not the number of waves.
constexpr int kBW = 8;            // waves per workgroup
constexpr int kBCH = 2;           // chunks per wave per segment (their activations stay in registers)
constexpr int kBSeg = kBW * kBCH; // chunks per segment (one pass of the workgroup over K)
// chunk `ch` of wave `wave` in segment `sg`: chunks go round the waves, so that a short last segment
// spreads over as many waves (and SIMDs) as it has chunks
template <int CH = 2>
__device__ __forceinline__ int wave_chunk(int sg, int wave, int ch) { return sg * (kBW * CH) + ch * kBW + wave; }
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
    float act_scale;              // 0: fp16 activations x/s; s_q > 0: INT8 codes of Sec. 4.1, output scaled by s_q
    int x_ready;                  // tokens kernel: x already holds the smoothed activations / the codes (transform_kernel)
    int wg_first;                 // first workgroup of this layer
};
// The table of first workgroups (wg_begin[1..16], 16 bits each) also travels as eight leading scalar
// kernel arguments: those are preloaded into scalar registers when a wave starts, so a workgroup
// knows its layer without a load and the problem record is the only load between the kernel's
// entry and its first index loads.  Number of table entries <= b, for b < 2^15 - 1:
struct WgTable { uint32_t t[kMaxGroup / 2]; };
__device__ __forceinline__ int layer_of_workgroup(uint32_t b, uint32_t t0, uint32_t t1, uint32_t t2, uint32_t t3,
                                                  uint32_t t4, uint32_t t5, uint32_t t6, uint32_t t7)
{
    // per 16-bit field f: bit 15 of (0x8000 + f) - (b + 1) is clear exactly when f <= b (no borrow crosses a field)
    const uint32_t bb = (b + 1u) * 0x00010001u, top = 0x80008000u;
    const uint32_t t[8] = {t0, t1, t2, t3, t4, t5, t6, t7};
    int n = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) n += __builtin_popcount(~((t[i] | top) - bb) & top);
    return n;
}
struct BucketBatch {
    BucketProblem p[kMaxGroup];
    int count;
};

// Walks the (visit, segment, tile) sequence of one workgroup.  Everything is wave-uniform.
// Padded (the tokens kernel): each (visit, segment) run is padded to a multiple of kSets steps so
// that the register-set rotation is static; padding steps load nothing and compute nothing.
// Unpadded (the bucket kernel): the sequence has real steps only and the kernel keeps track of the
// set a run starts with.
struct Cursor {
    int v0, v1, range_end, sg, i, steps;
    bool done, padded;
};

__device__ __forceinline__ int run_steps(const Cursor &c) { return c.padded ? (c.v1 - c.v0 + kSets - 1) / kSets * kSets : c.v1 - c.v0; }

template <bool PADDED>
__device__ __forceinline__ void cursor_begin(Cursor &c, int ta, int tb)
{
    c.padded = PADDED;
    c.v0 = ta; c.range_end = tb; c.v1 = min(tb, ta + kVisitTiles);
    c.sg = 0; c.i = 0; c.steps = run_steps(c); c.done = ta >= tb;
}

__device__ __forceinline__ void cursor_next_visit(Cursor &c)
{
    c.sg = 0; c.i = 0;
    if (c.v1 < c.range_end) {
        c.v0 = c.v1; c.v1 = min(c.range_end, c.v0 + kVisitTiles); c.steps = run_steps(c);
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
    uint4v cf;         // first step of a reduction group only: the lane's four per-bucket multipliers
};

// WITH_CF: this step opens a group of 16/NC row tiles that share one multiply-and-reduce; lane
// (bq, j) then also fetches the multipliers of rows 4bq..4bq+3, bucket j % NC, of the group's
// tile j / NC (fp32, accumulator order, straight from the table: every wave reads the same few
// hundred bytes, so they come from the L1/L2 cache).
// NC: accumulator columns one row tile uses; NB: per-bucket multipliers the table holds per row (NB < NC
// only with two tokens at 2 bits, where columns 4..7 are the second token's bucket sums and take the
// same multipliers as columns 0..3).
template <int NC, int NB = NC>
__device__ __forceinline__ uint4v load_multipliers(__amdgpu_buffer_rsrc_t rs_lut, int tile, int v1, int lane)
{
    const int j = lane & 15, bq = lane >> 4;
    const int t = tile + j / NC;
    return __builtin_amdgcn_raw_buffer_load_b128(rs_lut, t < v1 ? (uint32_t)((t * 4 + bq) * NB + (j % NB)) * 16 : kOob, 0, 0);
}

template <int BITS, bool WITH_CF, int MT = 1>
__device__ __forceinline__ void issue_step_loads(StepRegs<BITS> &r, const Cursor &c, __amdgpu_buffer_rsrc_t rs,
                                                 __amdgpu_buffer_rsrc_t rs_lut, int kc, int wave, int lane)
{
    constexpr uint32_t TB = BITS == 2 ? 1024 : 1536;
    constexpr int NB = BITS == 2 ? 4 : 8, NC = NB * MT;
    // a finished cursor or a padding step issues loads that are out of range: zeros, no traffic
    const int tile = c.v0 + c.i;
    const bool tv = !c.done && tile < c.v1;
#pragma unroll
    // the (tile, chunk) part of the address is wave-uniform and travels as the scalar offset, the
    // lane's part never changes; only the latter is range-checked, so an invalid step swaps it for
    // an offset that is out of range (and the scalar part for zero)
    for (int ch = 0; ch < kBCH; ++ch) {
        const int chunk = wave_chunk(c.sg, wave, ch);
        const bool v = tv && chunk < kc;
        const uint32_t o = v ? ((uint32_t)tile * (uint32_t)kc + (uint32_t)chunk) * TB : 0u;
        r.lo[ch] = __builtin_amdgcn_raw_buffer_load_b128(rs, v ? 16 * lane : kOob, o, kStreamPolicy);
        if (BITS == 3) r.hi[ch] = __builtin_amdgcn_raw_buffer_load_b64(rs, v ? 8 * lane : kOob, o + 1024, kStreamPolicy);
    }
    if (WITH_CF) r.cf = load_multipliers<NC, NB>(rs_lut, tile, c.done ? 0 : c.v1, lane);
}

// MT = 2 (2 bits only): two tokens.  The second token's activations take the place the sign-flipped
// activations have with 3 bits -- a second sparse pass over the same indices whose bucket sums land in
// columns 4..7 -- so the kernel has the 3-bit kernel's shape without its sign flips; columns 0..3 and
// 4..7 are multiplied by the same four centroids and reduced separately, one output per token.
//
// I8 (2 bits, activations quantised to the INT8 codes of Sec. 4.1): the codes travel as int8 numbers
// through v_smfmac_i32_16x16x128_i8, which takes all 16 two-bit fields of a packed word at once (stored
// byte e of a lane goes with field e, pairs of bytes share a group of four rows of B, and every fourth
// byte of B belongs to the same slot whichever lane holds it -- checked against a model on random data):
// half the matrix instructions and half the operand registers per weight.  The bucket sums are
// integers either way (exact in the fp32 accumulators of the fp16 route as well), so both routes give
// the same bits.
// NTOK: tokens the launch has (MT = 4 token slots also serve three tokens, which then leave the fourth pass out).
template <int BITS, int MT = 1, bool I8 = false, int NTOK = MT>
__global__ void __launch_bounds__(kBW * 64, 1) gemv_bucket_kernel(const uint32_t t0, const uint32_t t1, const uint32_t t2, const uint32_t t3,
                                                                   const uint32_t t4, const uint32_t t5, const uint32_t t6, const uint32_t t7,
                                                                   const BucketBatch batch)
{
    static_assert(MT == 1 || (MT == 2 && BITS == 2) || (MT == 4 && I8), "two tokens: 2-bit indices only; four: int8 operands only");
    static_assert(!I8 || BITS == 2 || MT == 1, "int8 operands: 2-bit indices, or one token at 3 bits");
    typedef int int4v __attribute__((ext_vector_type(4)));
    typedef int int8v __attribute__((ext_vector_type(8)));
    constexpr bool kHalfOps = !I8 || BITS == 3;  // fp16 operands kept (3 bits with int8 codes: for the sign-flipped pass)
    constexpr int NA = kHalfOps ? 8 : 1;         // fp16 operand registers (uint4) per chunk and token
    constexpr int NQ = I8 ? 4 : 1;               // int8 operand registers (uint4) per chunk and token
    constexpr int NB = BITS == 2 ? 4 : 8;        // buckets (centroids) per row
    constexpr int NC = NB * MT;                  // accumulator columns one row tile uses (MT > 1: 2 bits only)
    constexpr int TG = 16 / NC;                  // row tiles that share one reduction (4, 2 or 1)
    constexpr uint32_t TB = BITS == 2 ? 1024 : 1536;
    constexpr int NT = kBW * 64;
    constexpr int kSegHalfs = kBSeg * kTileCols;        // activations of one segment, one token
    constexpr int kPartFloats = kBW * kVisitTiles * 16; // the waves' partial outputs of one visit, one token
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS: [ xs: MT x one segment, kBSeg*256 halfs ][ part: MT x kBW*kVisitTiles*16 floats ][ 3 bits with int8 codes: one segment of bytes ]
    // (2 bits with int8 codes: the bytes take the place of the halfs)
    _Float16 *xs_lds = reinterpret_cast<_Float16 *>(smem);
    float *part = reinterpret_cast<float *>(smem + (size_t)MT * kSegHalfs * 2);
    uint8_t *xs8 = kHalfOps ? smem + (size_t)MT * kSegHalfs * 2 + (size_t)MT * kPartFloats * 4 : smem;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform: keeps addresses scalar
    const int q = lane >> 4, j = lane & 15, bq = lane >> 4;

    // which layer, which row tiles
    // (entries past the last layer hold the total, so they never count: no loop over `count`)
    const int pi = layer_of_workgroup(blockIdx.x, t0, t1, t2, t3, t4, t5, t6, t7);
    const BucketProblem pb = batch.p[pi];
    const int li = (int)blockIdx.x - pb.wg_first;
    const int ta = li * pb.tiles_base + min(li, pb.tiles_extra);
    const int tb = ta + pb.tiles_base + (li < pb.tiles_extra ? 1 : 0);
    const int kc = pb.kc, nseg = (kc + kBSeg - 1) / kBSeg;
    const bool quantised = pb.act_scale != 0.0f;               // wave-uniform
    const float out_scale = quantised ? pb.act_scale : 1.0f;
    const __amdgpu_buffer_rsrc_t rs_packed = make_rsrc(pb.packed, (uint32_t)pb.nt * (uint32_t)kc * TB);
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(pb.x, (uint32_t)NTOK * (uint32_t)kc * kTileCols * 2);
    const __amdgpu_buffer_rsrc_t rs_s = make_rsrc(pb.s, (uint32_t)kc * kTileCols * 4);
    const __amdgpu_buffer_rsrc_t rs_lut = make_rsrc(pb.lutA, (uint32_t)pb.nt * 16 * NB * 4);

    Cursor pf{}, cur{};
    cursor_begin<false>(pf, ta, tb);
    cur = pf;

    // Activations.  A segment is kBSeg*256 = 8 * (threads of the workgroup) columns, and thread t of
    // wave w smooths columns [8t, 8t+8) of it -- which lie in wave w's own two chunks.  So a wave
    // stages its activations through its own 1 KiB of LDS (to fan 8 values out to the 16 lanes
    // that need them) without any workgroup synchronisation.  The loads for a segment are issued
    // one segment ahead; the very first ones head the kernel, before the tile loads, because they
    // start the longest dependency chain.  Reads past the end of x / s return zero through the
    // buffer resource.
    uint4v xv[MT];
    float4v s0, s1;
    auto load_x = [&](int sg, bool valid) {
        const uint32_t g = (uint32_t)wave_chunk(sg, wave, lane >> 5) * 32 + (lane & 31);   // group of 8 columns
        valid = valid && g < (uint32_t)kc * 32;
#pragma unroll
        for (int t = 0; t < NTOK; ++t)   // token t's row of x starts K fp16 numbers after token t - 1's
            xv[t] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, valid ? g * 16 + (uint32_t)t * (uint32_t)kc * (kTileCols * 2) : kOob, 0, 0);
        s0 = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs_s, valid ? g * 32 : kOob, 0, 0));
        s1 = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs_s, valid ? g * 32 + 16 : kOob, 0, 0));
    };
    load_x(0, true);
    StepRegs<BITS> rs[kSets];   // always indexed by compile-time constants: four sets of registers
    issue_step_loads<BITS, true, MT>(rs[0], pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
    if (cur.done) return;   // no row tiles (the host never launches such a workgroup); the loads above moved nothing

    uint4v A[MT][kBCH][NA];   // this wave's smoothed activations of the current segment, NA operands per chunk and token
    uint4v Aq[MT][kBCH][NQ];  // I8: the codes as int8 numbers
    bool chunk_in_k[kBCH] = {};   // wave-uniform: a short last segment leaves some of the wave's chunks empty
    half16 B1;        // constant routing matrix (index c -> column c), built after the prologue
    int8v Bq[MT];     // I8: the same as int8 numbers; token t's sums go to columns 4t .. 4t+3
    float *my_part = part + wave * (kVisitTiles * 16);

    // bucket sums of one (tile, chunk): columns [0, NC) of a 16x16 accumulator
    auto tile_sums = [&](const StepRegs<BITS> &r) -> float4v {
        if constexpr (I8 && BITS == 3) {
            // the plain pass on int8 operands (4 instructions per chunk), the sign-flipped pass on fp16
            // operands as without I8 (8 per chunk): its flips are cheaper on fp16 numbers than on bytes
            int4v ax = {0, 0, 0, 0};
            float4v fy0 = {0.f, 0.f, 0.f, 0.f}, fy1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ch = 0; ch < kBCH; ++ch) {
                if (!chunk_in_k[ch]) continue;
                const unsigned long long h64 = ((unsigned long long)r.hi[ch][1] << 32) | r.hi[ch][0];
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const int idxreg = (int)r.lo[ch][d];
                    uint4v f0, f1;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int sh = 15 - (8 * (v >> 1) + 2 * d + (v & 1));
                        unsigned long long t = h64;
                        if (sh) asm("v_lshlrev_b64 %0, %1, %2" : "=v"(t) : "n"(sh), "v"(h64));
                        f0[v] = xor_and(A[0][ch][2 * d][v], (uint32_t)t, 0x80008000u);
                        f1[v] = xor_and(A[0][ch][2 * d + 1][v], (uint32_t)(t >> 32), 0x80008000u);
                    }
                    ax = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[0][ch][d]), Bq[0], ax, idxreg, 0, 0);
                    fy0 = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f0), B1, fy0, idxreg, 0, 0);
                    fy1 = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f1), B1, fy1, idxreg, 0, 1);
                }
            }
            float4v m;
#pragma unroll
            for (int u = 0; u < 4; ++u) m[u] = (float)ax[u] + dpp_f32<0x114>(fy0[u] + fy1[u]);   // flipped sums to columns 4..7
            return m;
        } else if constexpr (I8) {
            int4v ax = {0, 0, 0, 0}, ay = {0, 0, 0, 0}, az = {0, 0, 0, 0}, aw = {0, 0, 0, 0};
#pragma unroll
            for (int ch = 0; ch < kBCH; ++ch) {
                if (!chunk_in_k[ch]) continue;
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    const int idxreg = (int)r.lo[ch][d];
                    if (MT == 1) {
                        if (d & 1) ay = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[0][ch][d]), Bq[0], ay, idxreg, 0, 0);
                        else ax = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[0][ch][d]), Bq[0], ax, idxreg, 0, 0);
                    } else if (MT == 2) {
                        ax = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[0][ch][d]), Bq[0], ax, idxreg, 0, 0);
                        ay = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[MT - 1][ch][d]), Bq[MT - 1], ay, idxreg, 0, 0);
                    } else {   // four tokens: all routed to columns 0..3, moved apart below
                        ax = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[0][ch][d]), Bq[0], ax, idxreg, 0, 0);
                        ay = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[MT / 4][ch][d]), Bq[0], ay, idxreg, 0, 0);
                        az = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[MT / 2][ch][d]), Bq[0], az, idxreg, 0, 0);
                        if (NTOK > 3) aw = __builtin_amdgcn_smfmac_i32_16x16x128_i8(__builtin_bit_cast(int4v, Aq[MT - 1][ch][d]), Bq[0], aw, idxreg, 0, 0);
                    }
                }
            }
            float4v m;
#pragma unroll
            for (int u = 0; u < 4; ++u) {   // sums of at most 2^15 codes: exact
                int v = ax[u] + ay[u];
                if (MT == 4)   // tokens 1, 2, 3 to columns 4.., 8.., 12.. (row_shr:4 / 8 / 12; lanes shifted in read zero)
                    v = ax[u] + __builtin_amdgcn_update_dpp(0, ay[u], 0x114, 0xF, 0xF, true) + __builtin_amdgcn_update_dpp(0, az[u], 0x118, 0xF, 0xF, true) +
                        __builtin_amdgcn_update_dpp(0, aw[u], 0x11C, 0xF, 0xF, true);
                m[u] = (float)v;
            }
            return m;
        } else {
        float4v accx = {0.f, 0.f, 0.f, 0.f}, accy = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ch = 0; ch < kBCH; ++ch) {
            if (!chunk_in_k[ch]) continue;
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int idxreg = (int)r.lo[ch][d];
                // half a = 0 uses index bits [15:0], a = 1 bits [31:16]
                if (BITS == 2 && MT == 1) {
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[0][ch][2 * d]), B1, accx, idxreg, 0, 0);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[0][ch][2 * d + 1]), B1, accy, idxreg, 0, 1);
                } else if (BITS == 2) {   // two tokens: accx token 0, accy token 1
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[0][ch][2 * d]), B1, accx, idxreg, 0, 0);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[MT - 1][ch][2 * d]), B1, accy, idxreg, 0, 0);
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[0][ch][2 * d + 1]), B1, accx, idxreg, 0, 1);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[MT - 1][ch][2 * d + 1]), B1, accy, idxreg, 0, 1);
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
                        f0[v] = xor_and(A[0][ch][2 * d][v], (uint32_t)t, 0x80008000u);
                        f1[v] = xor_and(A[0][ch][2 * d + 1][v], (uint32_t)(t >> 32), 0x80008000u);
                    }
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[0][ch][2 * d]), B1, accx, idxreg, 0, 0);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f0), B1, accy, idxreg, 0, 0);
                    accx = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(A[0][ch][2 * d + 1]), B1, accx, idxreg, 0, 1);
                    accy = __builtin_amdgcn_smfmac_f32_16x16x64_f16(as_half8(f1), B1, accy, idxreg, 0, 1);
                }
            }
        }
        if (BITS == 2 && MT == 1) return accx + accy;
        // 3 bits: the sign-flipped sums move from columns 0..3 to columns 4..7 (two tokens: the second token's)
        float4v m;
#pragma unroll
        for (int u = 0; u < 4; ++u) m[u] = accx[u] + dpp_f32<0x114>(accy[u]);   // row_shr:4
        return m;
        }
    };

    // TG tiles share one multiply-and-reduce: tile u of the group moves to columns [u*NC, (u+1)*NC)
    auto reduce_group = [&](float4v m, int tl0, uint4v cfreg) {
#pragma clang fp contract(off)   // product, then lane-exchanging adds: fused into the product they cost an extra move each
        const int tl = tl0 + j / NC;                    // this lane's tile inside the visit
        const float4v cf = __builtin_bit_cast(float4v, cfreg);   // zeros past the end of the visit
        float4v pv;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float v = m[u] * cf[u];
            v += dpp_f32<kDppQuadXor1>(v);
            v += dpp_f32<kDppQuadXor2>(v);
            if (NC == 8 && MT == 1) v += dpp_f32<kDppRowHalfMirror>(v);
            asm volatile("" : "+v"(v));   // keeps the last add out of the branch below, where it could not take the lane exchange along
            pv[u] = v;
        }
        // one lane per (tile, token) holds the sum of its columns: two tokens keep columns 0..3 and 4..7 apart
        if ((j % (NC / MT)) == 0 && cur.v0 + tl < cur.v1) {
            float4v *slot = reinterpret_cast<float4v *>(&my_part[((j >> 2) & (MT - 1)) * kPartFloats + tl * 16 + 4 * bq]);
            if (cur.sg > 0) pv += *slot;
            *slot = pv;
        }
    };

    // Four steps = one turn of the register-set rotation: the step at position p uses set p and is
    // followed by the loads of the step three further on, into the set that position p - 1 has
    // just used.  The sequence of steps has no padding: a run (visit, segment) whose length is no
    // multiple of four ends in a shorter turn, after which the loads of the next run's first
    // three steps are under way in the sets behind its last step; the next run moves them to sets
    // 0..2 before its first turn (after the activations have been switched, so that they have had
    // that time to land) and fetches the multipliers of its first tiles again.  So the loads stay
    // three real steps ahead across segment and visit boundaries.
    StepRegs<BITS> &r0 = rs[0], &r1 = rs[1], &r2 = rs[2], &r3 = rs[3];
    const float4v zero = {0.f, 0.f, 0.f, 0.f};
    auto full_turn = [&]() __attribute__((always_inline)) {
        if constexpr (TG == 1) {   // every row tile has its own multipliers and its own reduction
            issue_step_loads<BITS, true, MT>(r3, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            float4v t = tile_sums(r0);
            uint4v cf = r0.cf;   // taken before the set is loaded again
            issue_step_loads<BITS, true, MT>(r0, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            reduce_group(t, cur.i, cf);
            t = tile_sums(r1); cf = r1.cf;
            issue_step_loads<BITS, true, MT>(r1, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            reduce_group(t, cur.i + 1, cf);
            t = tile_sums(r2); cf = r2.cf;
            issue_step_loads<BITS, true, MT>(r2, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            reduce_group(t, cur.i + 2, cf);
            t = tile_sums(r3);
            reduce_group(t, cur.i + 3, r3.cf);
            cur.i += 4;
            return;
        }
        float4v t0, t1, t3;
        issue_step_loads<BITS, false, MT>(r3, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
        t0 = tile_sums(r0);
        const uint4v cf_a = r0.cf;   // taken before the set is loaded again
        issue_step_loads<BITS, true, MT>(r0, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
        t1 = tile_sums(r1);
#pragma unroll
        for (int u = 0; u < 4; ++u) t0[u] += dpp_f32<(TG == 2 ? 0x118 : 0x114)>(t1[u]);   // row_shr:8 / row_shr:4
        if (TG == 2) reduce_group(t0, cur.i, cf_a);
        issue_step_loads<BITS, false, MT>(r1, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
        t1 = tile_sums(r2);
        const uint4v cf_b = r2.cf;
        issue_step_loads<BITS, TG == 2, MT>(r2, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
        t3 = tile_sums(r3);
        if (TG == 2) {
#pragma unroll
            for (int u = 0; u < 4; ++u) t1[u] += dpp_f32<0x118>(t3[u]);
            reduce_group(t1, cur.i + 2, cf_b);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                t1[u] += dpp_f32<0x114>(t3[u]);
                t0[u] += dpp_f32<0x118>(t1[u]);
            }
            reduce_group(t0, cur.i, cf_a);
        }
        cur.i += 4;
    };
    // the last 1..3 steps of a run (wave-uniform `left`): as many loads as steps
    auto short_turn = [&](int left) __attribute__((always_inline)) {
        if constexpr (TG == 1) {
            issue_step_loads<BITS, false, MT>(r3, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            float4v t = tile_sums(r0);
            reduce_group(t, cur.i, r0.cf);
            if (left > 1) {
                issue_step_loads<BITS, false, MT>(r0, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
                t = tile_sums(r1);
                reduce_group(t, cur.i + 1, r1.cf);
            }
            if (left > 2) {
                issue_step_loads<BITS, false, MT>(r1, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
                t = tile_sums(r2);
                reduce_group(t, cur.i + 2, r2.cf);
            }
            cur.i += 4;
            return;
        }
        float4v t0, t1 = zero;
        issue_step_loads<BITS, false, MT>(r3, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
        t0 = tile_sums(r0);
        const uint4v cf_a = r0.cf, cf_b = r2.cf;
        if (left > 1) {
            issue_step_loads<BITS, false, MT>(r0, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            t1 = tile_sums(r1);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) t0[u] += dpp_f32<(TG == 2 ? 0x118 : 0x114)>(t1[u]);
        if (TG == 2) reduce_group(t0, cur.i, cf_a);
        t1 = zero;
        if (left > 2) {
            issue_step_loads<BITS, false, MT>(r1, pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
            t1 = tile_sums(r2);
        }
        if (TG == 2) {
            if (left > 2) reduce_group(t1, cur.i + 2, cf_b);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) t0[u] += dpp_f32<0x118>(t1[u]);
            reduce_group(t0, cur.i, cf_a);
        }
        cur.i += 4;
    };
    int behind = 0;   // 1..3: the previous run ended in a short turn of that many steps (wave-uniform)
    // all turns of the run `cur` stands at
    auto run_turns = [&]() __attribute__((always_inline)) {
        if (behind) {
            // the next three steps' packed words sit in sets behind, behind + 1, behind + 2 (mod 4)
            auto take = [](StepRegs<BITS> &d, const StepRegs<BITS> &f) __attribute__((always_inline)) {
#pragma unroll
                for (int ch = 0; ch < kBCH; ++ch) { d.lo[ch] = f.lo[ch]; if (BITS == 3) d.hi[ch] = f.hi[ch]; }
            };
            if (behind == 1) { take(r0, r1); take(r1, r2); take(r2, r3); }
            else if (behind == 2) { StepRegs<BITS> t; take(t, r0); take(r0, r2); take(r1, r3); take(r2, t); }
            else { StepRegs<BITS> t, u; take(t, r0); take(u, r1); take(r0, r3); take(r1, t); take(r2, u); }
            r0.cf = load_multipliers<NC, NB>(rs_lut, cur.v0, cur.v1, lane);
            if (TG == 2) r2.cf = load_multipliers<NC, NB>(rs_lut, cur.v0 + 2, cur.v1, lane);
            if (TG == 1) {
                r1.cf = load_multipliers<NC, NB>(rs_lut, cur.v0 + 1, cur.v1, lane);
                r2.cf = load_multipliers<NC, NB>(rs_lut, cur.v0 + 2, cur.v1, lane);
            }
            behind = 0;
        }
        for (cur.i = 0; cur.i + 4 <= cur.steps;) full_turn();
        if (cur.i < cur.steps) { behind = cur.steps - cur.i; short_turn(behind); }
    };

    // the remaining two sets of the pipeline
    issue_step_loads<BITS, TG == 1, MT>(rs[1], pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
    issue_step_loads<BITS, TG <= 2, MT>(rs[2], pf, rs_packed, rs_lut, kc, wave, lane); cursor_advance(pf, nseg);
    while (!cur.done) {
        // (no workgroup synchronisation at the start of a visit: activations and multipliers are
        // per wave; the barrier that ends a visit's epilogue protects the reuse of `part`)
#pragma unroll
        for (int b = 0; b < 16; ++b) B1[b] = ((b & 3) == j) ? (_Float16)1.0f : (_Float16)0.0f;
        if constexpr (I8) {
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int b = 0; b < 8; ++b) Bq[t][b] = (j >> 2) == t ? 1 << (8 * (j & 3)) : 0;   // byte (b & 3) == j - 4t
        }
        for (cur.sg = 0; cur.sg < nseg; ++cur.sg) {
            {   // smooth this thread's 8 activations of the segment (loaded one segment ago)
                const bool in_k = wave_chunk(cur.sg, wave, lane >> 5) < kc;
#pragma unroll
                for (int t = 0; t < NTOK; ++t) {
                    half8 o;
                    if (!quantised) {
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            o[e] = !in_k ? (_Float16)0.0f : smooth_one((uint16_t)(xv[t][e >> 1] >> (16 * (e & 1))), e < 4 ? s0[e] : s1[e - 4]);
                    } else {   // wave-uniform branch
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            o[e] = !in_k ? (_Float16)0.0f
                                         : quantise_one((uint16_t)(xv[t][e >> 1] >> (16 * (e & 1))), make_divisor(e < 4 ? s0[e] : s1[e - 4], pb.act_scale));
                    }
                    if constexpr (I8) {   // the codes as int8 numbers, one byte per column
                        int c[8];
#pragma unroll
                        for (int e = 0; e < 8; ++e) c[e] = (int)(float)o[e] & 0xff;
                        const uint2v packed8 = {(uint32_t)(c[0] | c[1] << 8 | c[2] << 16 | c[3] << 24), (uint32_t)(c[4] | c[5] << 8 | c[6] << 16 | c[7] << 24)};
                        *reinterpret_cast<uint2v *>(xs8 + t * kSegHalfs + 8 * threadIdx.x) = packed8;
                    }
                    if constexpr (kHalfOps) *reinterpret_cast<half8 *>(&xs_lds[t * kSegHalfs + 8 * threadIdx.x]) = o;
                }
                // next segment's activations: of this visit, or segment 0 again for the next visit
                const bool more = cur.sg + 1 < nseg;
                load_x(more ? cur.sg + 1 : 0, more || cur.v1 < cur.range_end);
            }
#pragma unroll
            for (int ch = 0; ch < kBCH; ++ch) {
                chunk_in_k[ch] = wave_chunk(cur.sg, wave, ch) < kc;
#pragma unroll
                for (int t = 0; t < NTOK; ++t) {   // written by this wave only: no barrier
                    if constexpr (kHalfOps) {
#pragma unroll
                        for (int g = 0; g < 8; ++g)
                            A[t][ch][g] = *reinterpret_cast<const uint4v *>(&xs_lds[t * kSegHalfs + (wave * kBCH + ch) * kTileCols + 64 * q + 8 * g]);
                    }
                    if constexpr (I8) {
#pragma unroll
                        for (int g = 0; g < 4; ++g)
                            Aq[t][ch][g] = *reinterpret_cast<const uint4v *>(xs8 + t * kSegHalfs + (wave * kBCH + ch) * kTileCols + 64 * q + 16 * g);
                    }
                }
            }
            run_turns();
        }
        __syncthreads();
        // ---- visit epilogue: add the waves' slots in a fixed order, round once, store
        for (int e = threadIdx.x; e < (cur.v1 - cur.v0) * 16; e += NT) {
#pragma unroll
            for (int t = 0; t < NTOK; ++t) {   // token t's row of y starts N outputs after token t - 1's
                float sum = 0.f;
#pragma unroll
                for (int w = 0; w < kBW; ++w) sum += part[t * kPartFloats + w * (kVisitTiles * 16) + e];
                pb.y[(size_t)t * pb.nt * kTileRows + (size_t)cur.v0 * kTileRows + e] = __builtin_bit_cast(uint16_t, (_Float16)(sum * out_scale));
            }
        }
        cursor_next_visit(cur);
        if (!cur.done) __syncthreads();   // the next visit's waves overwrite their slots
    }
}


// ---- batched decode kernel (2 <= M <= 16): persistent workgroups over a group of layers -------
//
// Same walk as the bucket kernel (layer -> run of row tiles -> visits -> K segments -> steps, loads
// kSets-1 steps ahead), but the 16 columns of the matrix core's output tile are the tokens: the
// packed indices are dequantised in registers (v_perm_b32 through per-row byte-split codebook
// tables) into the A operand of v_mfma_f32_16x16x32_f16, and the smoothed activations of the
// wave's CH chunks, all tokens, stay in registers as B operands for a whole segment.
//   segment start  every wave smooths its own 512 columns of every token (Sec. 3.4: x / s) and
//                  fans them out to the B-operand layout through its own LDS stage: no workgroup
//                  synchronisation;
//   step           one row tile: 16 MFMAs per wave; after every second step the 8 waves' 16x16
//                  partial tiles of both meet in LDS (double-buffered, one s_barrier, no wait on
//                  outstanding loads) and the 512 threads add them in a fixed order.  With one segment the sum is rounded
//                  and stored; with several it accumulates in LDS until the last segment.
constexpr int kStageStride = kTileCols + 8;   // halfs per token row of a wave's stage (+16 B: no bank conflicts)

template <int BITS, int CH>
struct TokStepRegs {
    uint4v lo[CH];
    uint2v hi[CH];     // 3 bits: the third-bit words
    uint4v hi4[CH];    // 4 bits: the second plane
    uint4v tb;         // the lane's row of byte-split codebook tables (4 bits: the low bytes)
    uint4v tb2;        // 4 bits: the high bytes
};

template <int BITS, int CH>
__device__ __forceinline__ void issue_tok_loads(TokStepRegs<BITS, CH> &r, const Cursor &c, __amdgpu_buffer_rsrc_t rs,
                                                __amdgpu_buffer_rsrc_t rs_tb, int kc, int wave, int lane)
{
    constexpr uint32_t TB = kTileRows * kTileCols * BITS / 8;
    const int tile = c.v0 + c.i;
    const bool tv = !c.done && tile < c.v1;
#pragma unroll
    for (int ch = 0; ch < CH; ++ch) {
        const int chunk = wave_chunk<CH>(c.sg, wave, ch);
        const bool v = tv && chunk < kc;
        const uint32_t o = ((uint32_t)tile * (uint32_t)kc + (uint32_t)chunk) * TB;
        r.lo[ch] = __builtin_amdgcn_raw_buffer_load_b128(rs, v ? o + 16 * lane : kOob, 0, kStreamPolicy);
        if (BITS == 3) r.hi[ch] = __builtin_amdgcn_raw_buffer_load_b64(rs, v ? o + 1024 + 8 * lane : kOob, 0, kStreamPolicy);
        if (BITS == 4) r.hi4[ch] = __builtin_amdgcn_raw_buffer_load_b128(rs, v ? o + 1024 + 16 * lane : kOob, 0, kStreamPolicy);
    }
    const uint32_t row = (uint32_t)tile * kTileRows + (lane & 15);
    if (BITS == 2) {
        const uint2v t = __builtin_amdgcn_raw_buffer_load_b64(rs_tb, tv ? row * 8 : kOob, 0, 0);
        r.tb = uint4v{t[0], t[1], 0u, 0u};
    } else if (BITS == 3) {
        r.tb = __builtin_amdgcn_raw_buffer_load_b128(rs_tb, tv ? row * 16 : kOob, 0, 0);
    } else {
        r.tb = __builtin_amdgcn_raw_buffer_load_b128(rs_tb, tv ? row * 32 : kOob, 0, 0);
        r.tb2 = __builtin_amdgcn_raw_buffer_load_b128(rs_tb, tv ? row * 32 + 16 : kOob, 0, 0);
    }
}

template <int BITS, int CH>
__global__ void __launch_bounds__(kBW * 64, 1) gemv_tokens_kernel(const uint32_t t0, const uint32_t t1, const uint32_t t2, const uint32_t t3,
                                                                   const uint32_t t4, const uint32_t t5, const uint32_t t6, const uint32_t t7,
                                                                   const BucketBatch batch, const int M)
{
    constexpr int NC = BITS == 2 ? 4 : 8;
    constexpr uint32_t TB = kTileRows * kTileCols * BITS / 8;
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    // LDS: [ stage: kBW x 16 tokens x kStageStride halfs ][ red: 2 x 2 x kBW x 256 floats ][ sums: kVisitTiles x 256 floats ]
    _Float16 *stage = reinterpret_cast<_Float16 *>(smem) ;
    float *red = reinterpret_cast<float *>(smem + (size_t)kBW * 16 * kStageStride * 2);
    float *sums = red + 2 * 2 * kBW * 256;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int q = lane >> 4, j = lane & 15, bq = lane >> 4;

    const int pi = layer_of_workgroup(blockIdx.x, t0, t1, t2, t3, t4, t5, t6, t7);
    const BucketProblem pb = batch.p[pi];
    const int li = (int)blockIdx.x - pb.wg_first;
    const int ta = li * pb.tiles_base + min(li, pb.tiles_extra);
    const int tb_end = ta + pb.tiles_base + (li < pb.tiles_extra ? 1 : 0);
    const int kc = pb.kc, nseg = (kc + kBW * CH - 1) / (kBW * CH), K = kc * kTileCols, N = pb.nt * kTileRows;
    const bool x_ready = pb.x_ready != 0;                       // wave-uniform
    const float out_scale = pb.act_scale != 0.0f ? pb.act_scale : 1.0f;
    const __amdgpu_buffer_rsrc_t rs_packed = make_rsrc(pb.packed, (uint32_t)pb.nt * (uint32_t)kc * TB);
    const __amdgpu_buffer_rsrc_t rs_x = make_rsrc(pb.x, (uint32_t)M * (uint32_t)K * 2);
    const __amdgpu_buffer_rsrc_t rs_s = make_rsrc(pb.s, (uint32_t)K * 4);
    // byte-split tables: behind the bucket multipliers (2 and 3 bits), the whole table (4 bits)
    const __amdgpu_buffer_rsrc_t rs_tb = make_rsrc(reinterpret_cast<const uint8_t *>(pb.lutA) + (BITS == 4 ? 0 : (size_t)N * NC * 4),
                                                   (uint32_t)N * (BITS == 2 ? 8 : BITS == 3 ? 16 : 32));

    Cursor pf{}, cur{};
    cursor_begin<true>(pf, ta, tb_end);
    cur = pf;

    TokStepRegs<BITS, CH> r0, r1, r2, r3;
    uint4v Bx[CH][8];                      // B operands: lane (q, token j) holds 8 activations per MFMA
    bool chunk_in_k[CH] = {};                // wave-uniform: a short last segment leaves some chunks empty
    _Float16 *my_stage = stage + wave * (16 * kStageStride);

    // Smooth the wave's CH chunks of segment sg for all tokens and load them as B operands.
    // Lane l covers the 8 columns [8*(l&31), +8) of a chunk for the tokens 8*(l>>5) .. +7.
    uint4v xr[CH][8];
    float4v sa[CH], sb[CH];
    auto issue_activation_loads = [&](int sg) {
        const int kg = lane & 31, th = lane >> 5;
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            const int chunk = wave_chunk<CH>(sg, wave, ch);
            const uint32_t k0 = (uint32_t)chunk * kTileCols + 8 * kg;
            const bool cv = chunk < kc;
            sa[ch] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs_s, cv ? k0 * 4 : kOob, 0, 0));
            sb[ch] = __builtin_bit_cast(float4v, __builtin_amdgcn_raw_buffer_load_b128(rs_s, cv ? k0 * 4 + 16 : kOob, 0, 0));
#pragma unroll
            for (int mm = 0; mm < 8; ++mm) {
                const int m = th * 8 + mm;
                xr[ch][mm] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, (cv && m < M) ? ((uint32_t)m * (uint32_t)K + k0) * 2 : kOob, 0, 0);
            }
        }
    };
    auto finish_activations = [&](int sg) {
        const int kg = lane & 31, th = lane >> 5;
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            const bool cv = wave_chunk<CH>(sg, wave, ch) < kc;
            chunk_in_k[ch] = cv;
            // operand slot order 0,4,1,5,2,6,3,7 (the dequantiser pairs weight v with weight 4+v)
            if (!x_ready) {
                float rs[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) rs[e] = cv ? __builtin_amdgcn_rcpf(e < 4 ? sa[ch][e] : sb[ch][e - 4]) : 0.0f;
#pragma unroll
                for (int mm = 0; mm < 8; ++mm) {
                    const uint4v v = xr[ch][mm];   // register i: columns 2i, 2i+1; result register j: columns j, 4+j
                    uint4v o;
                    o[0] = smooth_pair<0, 0>(v[0], rs[0], v[2], rs[4]);
                    o[1] = smooth_pair<1, 1>(v[0], rs[1], v[2], rs[5]);
                    o[2] = smooth_pair<0, 0>(v[1], rs[2], v[3], rs[6]);
                    o[3] = smooth_pair<1, 1>(v[1], rs[3], v[3], rs[7]);
                    *reinterpret_cast<uint4v *>(&my_stage[(th * 8 + mm) * kStageStride + 8 * kg]) = o;
                }
            } else {   // wave-uniform branch: x already holds the operands, only the slot order is left
#pragma unroll
                for (int mm = 0; mm < 8; ++mm) {
                    const uint4v v = xr[ch][mm];   // OOB loads returned zero
                    uint4v o;
                    o[0] = __builtin_amdgcn_perm(v[2], v[0], 0x05040100u); o[1] = __builtin_amdgcn_perm(v[2], v[0], 0x07060302u);
                    o[2] = __builtin_amdgcn_perm(v[3], v[1], 0x05040100u); o[3] = __builtin_amdgcn_perm(v[3], v[1], 0x07060302u);
                    *reinterpret_cast<uint4v *>(&my_stage[(th * 8 + mm) * kStageStride + 8 * kg]) = o;
                }
            }
#pragma unroll
            for (int g = 0; g < 8; ++g)   // written by this wave only: LDS operations of a wave stay in order
                Bx[ch][g] = *reinterpret_cast<const uint4v *>(&my_stage[j * kStageStride + 64 * q + 8 * g]);
        }
    };

    auto tile_product = [&](const TokStepRegs<BITS, CH> &r) -> float4v {
        float4v acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        RowTables t;
        if (BITS == 2) { t.lo[0] = r.tb[0]; t.hi[0] = r.tb[1]; t.lo[1] = 0; t.hi[1] = 0; }
        else if (BITS == 4) { t.lo[0] = t.lo[1] = t.hi[0] = t.hi[1] = 0; }
        else { t.lo[0] = r.tb[0]; t.lo[1] = r.tb[1]; t.hi[0] = r.tb[2]; t.hi[1] = r.tb[3]; }
#pragma unroll
        for (int ch = 0; ch < CH; ++ch) {
            if (!chunk_in_k[ch]) continue;
            uint4v op0, op1;
            if (BITS == 4) {
                const RowTables4 t4{{r.tb[0], r.tb[1], r.tb[2], r.tb[3]}, {r.tb2[0], r.tb2[1], r.tb2[2], r.tb2[3]}};
#pragma unroll
                for (int d = 0; d < 4; ++d) {
                    decode_word4(r.lo[ch][d], r.hi4[ch][d], t4, op0, op1);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op0), as_half8(Bx[ch][2 * d]), acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op1), as_half8(Bx[ch][2 * d + 1]), acc1, 0, 0, 0);
                }
                continue;
            }
            HighBits hb{0u, 0u};
            if (BITS == 3) hb = regroup_high(r.hi[ch]);
            decode_word<BITS, 0>(r.lo[ch][0], hb, t, op0, op1);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op0), as_half8(Bx[ch][0]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op1), as_half8(Bx[ch][1]), acc1, 0, 0, 0);
            decode_word<BITS, 1>(r.lo[ch][1], hb, t, op0, op1);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op0), as_half8(Bx[ch][2]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op1), as_half8(Bx[ch][3]), acc1, 0, 0, 0);
            decode_word<BITS, 2>(r.lo[ch][2], hb, t, op0, op1);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op0), as_half8(Bx[ch][4]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op1), as_half8(Bx[ch][5]), acc1, 0, 0, 0);
            decode_word<BITS, 3>(r.lo[ch][3], hb, t, op0, op1);
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op0), as_half8(Bx[ch][6]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(as_half8(op1), as_half8(Bx[ch][7]), acc1, 0, 0, 0);
        }
        return acc0 + acc1;   // lane (bq, j): rows 4bq..4bq+3 of token j
    };

    // two steps: this wave's two partial tiles -> LDS; one barrier; every thread adds one output of
    // one of the two tiles over the waves, in a fixed order
    int phase = 0;
    auto finish_pair = [&](float4v p0, float4v p1, int tl, bool second) {
        float *buf = red + phase * (2 * kBW * 256);
        *reinterpret_cast<float4v *>(&buf[wave * 256 + j * 16 + 4 * bq]) = p0;
        *reinterpret_cast<float4v *>(&buf[(kBW + wave) * 256 + j * 16 + 4 * bq]) = p1;
        // LDS writes done, then the barrier; outstanding global loads keep flying
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const int which = threadIdx.x >> 8, o = threadIdx.x & 255;   // waves 0-3: first tile, waves 4-7: second
        if (which == 0 || second) {
            const int m = o >> 4, row = o & 15;
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < kBW; ++w) sum += buf[(which * kBW + w) * 256 + o];
            if (nseg > 1) {
                float *slot = &sums[(tl + which) * 256 + o];
                if (cur.sg > 0) sum += *slot;
                if (cur.sg + 1 < nseg) *slot = sum;
            }
            if (cur.sg + 1 == nseg && m < M)
                pb.y[(size_t)m * N + (size_t)(cur.v0 + tl + which) * kTileRows + row] = __builtin_bit_cast(uint16_t, (_Float16)(sum * out_scale));
        }
        phase ^= 1;
    };

    auto four_steps = [&]() {
        const int left = (cur.v1 - cur.v0) - cur.i;   // tiles left in this run; padding steps skip their work
        const float4v zero = {0.f, 0.f, 0.f, 0.f};
        float4v p0, p1 = zero;
        issue_tok_loads<BITS, CH>(r3, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
        p0 = tile_product(r0);
        issue_tok_loads<BITS, CH>(r0, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
        if (left > 1) p1 = tile_product(r1);
        finish_pair(p0, p1, cur.i, left > 1);
        issue_tok_loads<BITS, CH>(r1, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
        p1 = zero;
        if (left > 2) p0 = tile_product(r2);
        issue_tok_loads<BITS, CH>(r2, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
        if (left > 3) p1 = tile_product(r3);
        if (left > 2) finish_pair(p0, p1, cur.i + 2, left > 3);
        cur.i += 4;
    };

    issue_activation_loads(0);   // they start the longest dependency chain: ahead of the tile loads
    issue_tok_loads<BITS, CH>(r0, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
    issue_tok_loads<BITS, CH>(r1, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
    issue_tok_loads<BITS, CH>(r2, pf, rs_packed, rs_tb, kc, wave, lane); cursor_advance(pf, nseg);
    if (cur.done) return;   // no row tiles (the host never launches such a workgroup); the loads above moved nothing
    finish_activations(0);
    bool primed = true;   // the first segment's activations are in place
    while (!cur.done) {
        for (cur.sg = 0; cur.sg < nseg; ++cur.sg) {
            if (!primed) {
                issue_activation_loads(cur.sg);
                finish_activations(cur.sg);
            }
            primed = false;
            for (cur.i = 0; cur.i < cur.steps;) four_steps();
        }
        cursor_next_visit(cur);
    }
}

// ---- activation transformation ahead of the tokens kernel (Sec. 4.1) -----------------------------
// On the tokens kernel's route (2..16 tokens, and 4 bits) every workgroup of a layer stages the whole activation matrix, so whatever is
// done to an activation is repeated by each of them.  This small kernel does it once per layer
// and leaves the result, as fp16 numbers in the layout of x, in the workspace: the INT8 codes of
// Eq. 10 (always: the divisions are expensive), or the smoothed activations x/s when K is large
// enough for the saving to exceed the extra launch.  One thread takes 8 columns of a few tokens:
// the divisor-only part of the division is shared by them.
struct TransformItem {
    const uint16_t *x;
    const float *s;
    uint16_t *codes;
    int K;
    float s_q;
};
struct TransformBatch {
    TransformItem p[kMaxGroup];
};
constexpr int kQuantThreads = 64;
constexpr int kQuantTokens = 4;
constexpr int kPrepassMinK = 16384;   // widest layer of a group from which fp16 activations are smoothed ahead

__global__ __launch_bounds__(kQuantThreads) void transform_kernel(TransformBatch batch, int M)
{
    const TransformItem it = batch.p[blockIdx.y];
    const int k0 = ((int)blockIdx.x * kQuantThreads + (int)threadIdx.x) * 8;
    if (k0 >= it.K) return;   // K is a multiple of 256: a thread's 8 columns are all inside or all outside
    const float4v s0 = *reinterpret_cast<const float4v *>(it.s + k0), s1 = *reinterpret_cast<const float4v *>(it.s + k0 + 4);
    const bool quantised = it.s_q != 0.0f;   // uniform
    Divisor dv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) dv[e] = make_divisor(e < 4 ? s0[e] : s1[e - 4], quantised ? it.s_q : 1.0f);
    // blockIdx.z: a group of kQuantTokens tokens (short dependent chains, all loads in flight together)
    const int m0 = (int)blockIdx.z * kQuantTokens;
    uint4v v[kQuantTokens];
#pragma unroll
    for (int i = 0; i < kQuantTokens; ++i)
        if (m0 + i < M) v[i] = *reinterpret_cast<const uint4v *>(it.x + (size_t)(m0 + i) * it.K + k0);
#pragma unroll
    for (int i = 0; i < kQuantTokens; ++i) {
        if (m0 + i < M) {
            half8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint16_t xb = (uint16_t)(v[i][e >> 1] >> (16 * (e & 1)));
                if (quantised) o[e] = quantise_one(xb, dv[e]);
                else o[e] = smooth_one(xb, e < 4 ? s0[e] : s1[e - 4]);   // rounds as the fused path does
            }
            *reinterpret_cast<half8 *>(it.codes + (size_t)(m0 + i) * it.K + k0) = o;
        }
    }
}

// compute units of the current device (looked up once per device)
static int num_cus()
{
    static std::atomic<int> cus[kMaxDevices] = {};
    const int dev = current_device();
    if (dev < 0) return 256;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// One launch for a group of decode problems: the bucket kernel for one token, the tokens kernel for 2..16.
int launch_decode_group(const GroupItem *items, int count, int M, int bits, void *workspace, void *stream_, bool force_prepass)
{
    hipStream_t stream = (hipStream_t)stream_;
    BucketBatch batch{};
    int tiles = 0;
    // 4 bits: the register dequantiser serves one token too; 2 bits: the sparse-matrix-core kernel also takes
    // two tokens (one sparse pass per token costs less than dequantising once)
    // (with the INT8 codes of Sec. 4.1 as int8 operands the sparse-matrix-core kernel has room for four tokens)
    bool all_quantised = true;
    for (int i = 0; i < count; ++i) all_quantised = all_quantised && items[i].act_scale != 0.0f;
    const int sparse_tokens = bits != 2 ? 1 : all_quantised ? 4 : 2;   // most tokens the bucket kernel takes
    const bool tokens_path = bits == 4 || M > sparse_tokens;
    const int MT = M <= 2 ? M : 4;                                      // token slots of the bucket kernel variant
    // several tokens: quantised activations are made once, ahead of the product, and so are smoothed
    // ones when the layers are wide (measured: the launch costs about 3.6 us; re-smoothing in every
    // workgroup costs 1.9 us for K = 4096 / 11008 and 4.3 us for K = 8192 / 28672)
    const uint16_t *codes[kMaxGroup] = {};
    int widest = 0;
    for (int i = 0; i < count; ++i) widest = items[i].K > widest ? items[i].K : widest;
    if (tokens_path && (force_prepass || items[0].act_scale != 0.0f || widest >= kPrepassMinK)) {
        // layers that read the same input (same x, s, K and quantisation step: q/k/v or gate/up of a decoder
        // block) share one transformed copy
        TransformBatch qb{};
        size_t offset = 0;
        int max_k = 0, distinct = 0;
        for (int i = 0; i < count; ++i) {
            for (int d = 0; d < distinct && !codes[i]; ++d)
                if (qb.p[d].x == items[i].x && qb.p[d].s == items[i].s && qb.p[d].K == items[i].K && qb.p[d].s_q == items[i].act_scale)
                    codes[i] = qb.p[d].codes;
            if (codes[i]) continue;
            uint16_t *dst = reinterpret_cast<uint16_t *>(static_cast<char *>(workspace) + offset);
            qb.p[distinct++] = TransformItem{items[i].x, items[i].s, dst, items[i].K, items[i].act_scale};
            codes[i] = dst;
            offset += decode_codes_bytes(M, items[i].K);
            if (items[i].K > max_k) max_k = items[i].K;
        }
        const int per_block = kQuantThreads * 8;
        void *qargs[] = {&qb, const_cast<int *>(&M)};
        if (hipError_t e = hipLaunchKernel((const void *)transform_kernel, dim3((max_k + per_block - 1) / per_block, distinct, (M + kQuantTokens - 1) / kQuantTokens),
                                           dim3(kQuantThreads), qargs, 0, stream)) return (int)e;
    }
    for (int i = 0; i < count; ++i) {
        BucketProblem &p = batch.p[i];
        p.packed = (const uint8_t *)items[i].packed;
        p.lutA = (const float *)items[i].lut;
        p.x = codes[i] ? codes[i] : items[i].x; p.s = items[i].s; p.y = items[i].y;
        p.nt = items[i].N / kTileRows; p.kc = items[i].K / kTileCols;
        p.act_scale = items[i].act_scale;
        p.x_ready = codes[i] != nullptr;
        tiles += p.nt;
    }
    // Workgroups per layer.  A layer's time is that of its slowest workgroup, in units of two-chunk
    // steps: a fixed start-up, then for each K segment one pass over its row tiles plus the cost of
    // switching to the segment's activations.  A wave takes `ch` chunks of a full segment; a short
    // last segment gives every wave ceil(rest / 8).  The split minimises the time of the slowest layer.
    int grid = num_cus();
    if (grid > tiles) grid = tiles;
    if (grid < count) grid = count;
    // 2 bits on the sparse matrix core with quantised activations: the codes go in as int8 numbers
    const bool int8_codes = !tokens_path && bits != 4 && all_quantised;   // (3 bits: one token, the plain pass only)
    const bool light_steps = !tokens_path && bits == 2 && M == 1;   // one sparse pass per tile: a step is short next to the fixed costs
    // the several-token kernel, measured per workgroup (unit: the time of two chunks of one row tile, about 1 us):
    // smoothing inside the kernel, a segment switch re-stages 16 tokens x 512 columns per wave (2.3); with the
    // activations transformed ahead it only permutes them (1.5)
    const bool staged_ahead = tokens_path && codes[0] != nullptr;
    const double startup_steps = tokens_path ? (staged_ahead ? 0.5 : 0.7) : light_steps ? 3.5 : 2.0;
    const double segment_steps = tokens_path ? (staged_ahead ? 1.5 : 2.3) : light_steps ? 1.8 : 0.4;
    const double step_overhead = tokens_path ? (staged_ahead ? 0.22 : 0.3) : 0.1;   // per tile and segment: barrier / bookkeeping
    auto layer_time_with = [&](int ch, int i, int n) {
        const int seg = kBW * ch;
        const int kc = batch.p[i].kc, segs = (kc + seg - 1) / seg, rest = kc % seg;
        const double steps_per_tile = (kc / seg) * (0.5 * ch + step_overhead) +
                                      (rest ? 0.5 * ((rest + kBW - 1) / kBW) + step_overhead : 0.0);
        const int t = (batch.p[i].nt + n - 1) / n, visits = (t + kVisitTiles - 1) / kVisitTiles;
        return startup_steps + steps_per_tile * t + segs * visits * segment_steps;
    };
    auto split = [&](int ch, int *nwg) {
        auto layer_time = [&](int i, int n) { return layer_time_with(ch, i, n); };
        // smallest number of workgroups with which layer i takes at most T (0: not even one per tile does)
        auto need = [&](int i, double T) {
            const int nt = batch.p[i].nt;
            if (layer_time(i, nt) > T) return 0;
            int lo = 1, hi = nt;               // layer_time never grows with n
            while (lo < hi) {
                const int mid = (lo + hi) / 2;
                if (layer_time(i, mid) <= T) hi = mid; else lo = mid + 1;
            }
            return lo;
        };
        auto fits = [&](double T, int *out) {
            int sum = 0;
            for (int i = 0; i < count; ++i) {
                const int n = need(i, T);
                if (n == 0) return false;
                out[i] = n;
                sum += n;
            }
            return sum <= grid;
        };
        // the smallest common finish time the grid can reach: bisection over T between "one workgroup per
        // tile everywhere" and "one workgroup per layer" (the host guarantees grid >= count)
        double t_lo = 0.0, t_hi = 0.0;
        for (int i = 0; i < count; ++i) {
            t_lo = std::max(t_lo, layer_time(i, batch.p[i].nt));
            t_hi = std::max(t_hi, layer_time(i, 1));
        }
        int trial[kMaxGroup];
        if (fits(t_lo, trial)) t_hi = t_lo;
        for (int it = 0; it < 24 && t_hi - t_lo > 0.02; ++it) {
            const double mid = 0.5 * (t_lo + t_hi);
            if (fits(mid, trial)) t_hi = mid; else t_lo = mid;
        }
        fits(t_hi, nwg);
        int used = 0;
        for (int i = 0; i < count; ++i) used += nwg[i];
        while (used < grid) {                  // spare workgroups: one by one to the layer that is slowest then
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
    };
    // the split depends on the shapes only: the last one is kept (serving loops repeat a few groups)
    struct SplitMemo { int count, M, bits, grid, ahead, route, nt[kMaxGroup], kc[kMaxGroup], nwg[kMaxGroup]; };
    static thread_local SplitMemo memo = {};
    const int route = tokens_path ? 1 : int8_codes ? 2 : 0;   // the cost constants depend on it
    bool known = memo.count == count && memo.M == M && memo.bits == bits && memo.grid == grid && memo.ahead == (int)staged_ahead && memo.route == route;
    for (int i = 0; known && i < count; ++i) known = memo.nt[i] == batch.p[i].nt && memo.kc[i] == batch.p[i].kc;
    int nwg[kMaxGroup];
    if (known) {
        for (int i = 0; i < count; ++i) nwg[i] = memo.nwg[i];
    } else {
        split(kBCH, nwg);
        memo.count = count; memo.M = M; memo.bits = bits; memo.grid = grid; memo.ahead = (int)staged_ahead; memo.route = route;
        for (int i = 0; i < count; ++i) { memo.nt[i] = batch.p[i].nt; memo.kc[i] = batch.p[i].kc; memo.nwg[i] = nwg[i]; }
    }
    // Workgroups are dispatched in the order of their ids, the last of a full grid almost 1 us after the
    // first: the layers whose workgroups have the most to do take the lowest ids.
    {
        int order[kMaxGroup];
        double t[kMaxGroup];
        for (int i = 0; i < count; ++i) { order[i] = i; t[i] = layer_time_with(kBCH, i, nwg[i]); }
        std::stable_sort(order, order + count, [&](int a, int b) { return t[a] > t[b]; });
        BucketProblem sorted_p[kMaxGroup];
        int sorted_n[kMaxGroup];
        for (int q = 0; q < count; ++q) { sorted_p[q] = batch.p[order[q]]; sorted_n[q] = nwg[order[q]]; }
        for (int q = 0; q < count; ++q) { batch.p[q] = sorted_p[q]; nwg[q] = sorted_n[q]; }
    }
    grid = 0;
    for (int i = 0; i < count; ++i) grid += nwg[i];
    int acc = 0;
    int wg_begin[kMaxGroup + 1];   // first workgroup of every layer; entries past the last layer hold the total
    for (int i = 0; i < count; ++i) {
        wg_begin[i] = acc;
        acc += nwg[i];
        batch.p[i].tiles_base = batch.p[i].nt / nwg[i];
        batch.p[i].tiles_extra = batch.p[i].nt % nwg[i];
    }
    for (int i = count; i <= kMaxGroup; ++i) wg_begin[i] = acc;
    batch.count = count;
    static_assert(kMaxGroup == 16, "eight leading kernel arguments hold wg_begin[1..16]");
    if (acc >= 0x7fff) return (int)hipErrorInvalidConfiguration;   // 16-bit table fields (acc <= max(CUs, count))
    WgTable table;
    for (int i = 0; i < kMaxGroup / 2; ++i) table.t[i] = (uint32_t)wg_begin[2 * i + 1] | (uint32_t)wg_begin[2 * i + 2] << 16;
    for (int i = 0; i < count; ++i) batch.p[i].wg_first = wg_begin[i];
    const int NC = bits == 2 ? 4 : 8;
    size_t lds;
    const void *fn;
    if (!tokens_path) {
        lds = (size_t)MT * ((size_t)kBSeg * kTileCols * 2 + (size_t)kBW * kVisitTiles * 16 * 4) + (bits == 3 && int8_codes ? (size_t)kBSeg * kTileCols : 0);
        fn = bits == 3 ? (int8_codes ? (const void *)gemv_bucket_kernel<3, 1, true> : (const void *)gemv_bucket_kernel<3>)
             : int8_codes ? (MT == 4 ? (M == 3 ? (const void *)gemv_bucket_kernel<2, 4, true, 3> : (const void *)gemv_bucket_kernel<2, 4, true>)
                             : MT == 2 ? (const void *)gemv_bucket_kernel<2, 2, true> : (const void *)gemv_bucket_kernel<2, 1, true>)
             : MT == 2 ? (const void *)gemv_bucket_kernel<2, 2> : (const void *)gemv_bucket_kernel<2>;
    } else {
        lds = (size_t)kBW * 16 * kStageStride * 2 + (size_t)2 * 2 * kBW * 256 * 4 + (size_t)kVisitTiles * 256 * 4;
        fn = bits == 2 ? (const void *)gemv_tokens_kernel<2, kBCH> : bits == 3 ? (const void *)gemv_tokens_kernel<3, kBCH>
                                                                              : (const void *)gemv_tokens_kernel<4, kBCH>;
    }
    static PerDeviceFlags<21> lds_raised;   // (variant 3 at 3 bits is the kernel with the int8 plain pass)
    const int variant = tokens_path ? 1 : int8_codes ? (MT == 4 ? (M == 3 ? 6 : 5) : MT == 2 ? 4 : 3) : MT == 2 ? 2 : 0;
    if (hipError_t e = raise_lds_limit_once(lds_raised, variant * 3 + (bits - 2), fn, lds)) return (int)e;
    void *args[] = {&table.t[0], &table.t[1], &table.t[2], &table.t[3], &table.t[4], &table.t[5], &table.t[6], &table.t[7],
                    &batch, const_cast<int *>(&M)};   // the bucket kernel takes no M
    if (hipError_t e = hipLaunchKernel(fn, dim3(grid), dim3(kBW * 64), args, lds, stream)) return (int)e;
    return (int)hipGetLastError();
}

// ---- scratch for callers that cannot allocate ---------------------------------------------------
// lcd_lut_gemv_noalloc keeps the transformed activations (at most 16 tokens x kStaticScratchCols
// columns, fp16) in this file-scope device array instead of a workspace the caller brings.  Every GPU
// holds its own copy at its own address; the array's name is only a host-side handle, so the device
// address is asked for once per device and kernels are given that address.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// Device address of the current device's scratch array (hipError_t as int; 0 = success).
static int static_scratch(void **out)
{
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev)) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return 0;
}

int launch_gemv_noalloc(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                        int M, int N, int K, int bits, void *stream_)
{
    void *ws = nullptr;
    if (int e = static_scratch(&ws)) return e;
    GroupItem it{packed, lut, x, s, y, N, K, 0.0f};
    // the activations always go through the scratch array on the several-token route, whatever K is
    return launch_decode_group(&it, 1, M, bits, ws, stream_, true);
}

int launch_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, float act_scale, void *workspace, void *stream_)
{
    GroupItem it{packed, lut, x, s, y, N, K, act_scale};
    return launch_decode_group(&it, 1, M, bits, workspace, stream_, false);
}

}  // namespace lcd
