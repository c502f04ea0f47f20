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

inline size_t tile_bytes(int bits) { return (size_t)kTileRows * kTileCols * bits / 8; }   // 1024, 1536, 2048

lcd_status fail(lcd_status st, const char *fmt, ...);

struct GemmPlan {
    int m_pad;             // tokens rounded up to the workgroup tile (128)
    size_t xs_bytes;       // workspace: smoothed activations fp16, operand order, m_pad x K
};
GemmPlan plan_gemm(int M, int N, int K, int bits);

constexpr int kMaxGroup = 16;     // problems per grouped launch

struct GroupItem {
    const void *packed; const void *lut; const uint16_t *x; const float *s; uint16_t *y; int N, K;
    float act_scale;   // 0: fp16 activations; s_q > 0: INT8 activation codes (paper Sec. 4.1)
};
// one launch for `count` decode problems (1 <= M <= 16 tokens each)
// (workspace: decode_codes_bytes(M, K) per item, in item order, when M > 1 and act_scale != 0)
// force_prepass: the activations are transformed ahead of the product (into the workspace) whenever the
// several-token kernel runs, not only where that is the faster route
int launch_decode_group(const GroupItem *items, int count, int M, int bits, void *workspace, void *stream, bool force_prepass = false);
inline size_t decode_codes_bytes(int M, int K) { return ((size_t)M * K * 2 + 255) / 256 * 256; }

// Launchers implemented in the .hip files.  All return hipError_t as int (0 = success).
int launch_pack(const uint8_t *idx, int N, int K, int bits, void *packed, void *stream);
int launch_unpack(const void *packed, int N, int K, int bits, uint8_t *idx, void *stream);
int launch_build_lut(const uint16_t *codebook, int N, int bits, void *lut, void *stream);
int launch_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, float act_scale, void *workspace, void *stream);
// the same product with the library's own static device array as the workspace (no allocation anywhere)
constexpr int kStaticScratchCols = 32768;                                   // largest K at 16 tokens
constexpr size_t kStaticScratchBytes = (size_t)16 * kStaticScratchCols * 2;  // 1 MiB per GPU
int launch_gemv_noalloc(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                        int M, int N, int K, int bits, void *stream);
int launch_gemm(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                int M, int N, int K, int bits, float act_scale, void *workspace, const GemmPlan &plan, void *stream);
int launch_assign(const uint16_t *w, const uint16_t *codebook, int ncent, int N, int K, int bits, uint8_t *idx, void *stream);
int launch_counts(const uint8_t *idx, int N, int K, int bits, uint32_t *counts, void *stream);
int launch_merge(const uint16_t *cb_in, const uint32_t *counts, const uint8_t *idx_in, int ncent, int N, int K, int bits,
                 uint16_t *cb_out, uint8_t *idx_out, uint8_t *merged, void *stream);
const char *hip_error_name(int err);
// s_q = 0: xs = x / s; s_q > 0: the INT8 codes of Sec. 4.1 (as fp16 numbers)
int launch_smooth(const uint16_t *x, const float *s, void *xs, int M, int Mpad, int K, float s_q, void *stream);
struct SmoothItem { const uint16_t *x; const float *s; void *xs; int K; float s_q; };
int launch_smooth_group(const SmoothItem *items, int count, int M, int Mpad, void *stream);
// prefill, several layers in one launch; the workspace holds every layer's smoothed activations side by side
int launch_gemm_group(const GroupItem *items, int count, int M, int bits, void *workspace, void *stream);

}  // namespace lcd
