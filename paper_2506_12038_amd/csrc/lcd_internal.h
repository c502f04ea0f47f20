// Internal declarations shared by the host-side C ABI and the HIP kernels' launchers.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include "lcd.h"

#define LCD_VERSION 100
#define LCD_LAYOUT_REVISION 1

namespace lcd {

constexpr int kTileRows = 16;    // rows of the index matrix per tile
constexpr int kTileCols = 256;   // columns per tile (one 16-byte load per lane of a wave)
constexpr int kLaneCols = 64;    // columns one lane's 128-bit word covers

inline size_t tile_bytes(int bits) { return bits == 2 ? 1024 : 1536; }

lcd_status fail(lcd_status st, const char *fmt, ...);

// How lcd_lut_gemv splits one problem over the chip.  Pure host arithmetic.
struct GemvPlan {
    int ch;                // 256-column chunks whose activations one wave keeps in registers
    int waves;             // waves per workgroup (each owns `ch` consecutive chunks)
    int splits;            // workgroups along K (partials are reduced by a second kernel if > 1)
    int chunks_per_split;  // waves * ch
    int grid_x;            // workgroups along N (each loops over row tiles with this stride)
    size_t xs_bytes;       // workspace: smoothed activations fp16 [M][K] (batched path only)
    size_t partial_bytes;  // workspace: fp32 partial sums [splits][M][N] (splits > 1 only)
};
GemvPlan plan_gemv(int M, int N, int K, int bits);

struct GemmPlan {
    int m_pad;             // tokens rounded up to the workgroup tile (128)
    size_t xs_bytes;       // workspace: smoothed activations fp16, operand order, m_pad x K
};
GemmPlan plan_gemm(int M, int N, int K, int bits);

constexpr int kMaxGroup = 16;     // problems per grouped launch

struct GroupItem {
    const void *packed; const void *lut; const uint16_t *x; const float *s; uint16_t *y; int N, K;
};
int launch_bucket_group(const GroupItem *items, int count, int bits, void *stream);

// Launchers implemented in the .hip files.  All return hipError_t as int (0 = success).
int launch_pack(const uint8_t *idx, int N, int K, int bits, void *packed, void *stream);
int launch_unpack(const void *packed, int N, int K, int bits, uint8_t *idx, void *stream);
int launch_build_lut(const uint16_t *codebook, int N, int bits, void *lut, void *stream);
int launch_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, void *workspace, const GemvPlan &plan, void *stream);
int launch_gemm(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, void *workspace, const GemmPlan &plan, void *stream);
const char *hip_error_name(int err);
int launch_smooth(const uint16_t *x, const float *s, void *xs, int M, int Mpad, int K, int layout, void *stream);
int launch_reduce(const float *partial, uint16_t *y, int splits, long long total, void *stream);

}  // namespace lcd
