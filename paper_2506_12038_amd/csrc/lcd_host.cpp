// Host side of the C ABI: argument validation, error strings, size arithmetic and the host
// twins of the index packer.  Nothing here touches the GPU.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>
#include "lcd_internal.h"

namespace lcd {

static thread_local char g_err[512] = "";

lcd_status fail(lcd_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

static lcd_status check_shape(int N, int K, int bits)
{
    if (bits < 2 || bits > 4) return fail(LCD_ERR_BAD_BITS, "bits=%d: only 2, 3 and 4 are supported", bits);
    if (N <= 0 || K <= 0 || N % kTileRows != 0 || K % kTileCols != 0)
        return fail(LCD_ERR_BAD_SHAPE, "N=%d must be a positive multiple of %d and K=%d of %d", N, kTileRows, K, kTileCols);
    if ((long long)N * (long long)K * bits / 8 >= (1ll << 32)) return fail(LCD_ERR_BAD_SHAPE, "packed matrix must be smaller than 4 GiB");
    return LCD_OK;
}

static lcd_status check_aligned(const void *p, const char *name)
{
    if (!p) return fail(LCD_ERR_NULL, "%s is NULL", name);
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0) return fail(LCD_ERR_ALIGN, "%s is not 16-byte aligned", name);
    return LCD_OK;
}

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

GemmPlan plan_gemm(int M, int N, int K, int bits)
{
    (void)N; (void)bits;
    GemmPlan p{};
    p.m_pad = (M + 127) / 128 * 128;
    p.xs_bytes = round_up((size_t)p.m_pad * K * 2, 256);
    return p;
}

// ---- host packer: walks tiles and lanes, builds each lane's words -----------------------
static void lane_words(const uint8_t *row64, int bits, uint32_t lo[4], uint32_t hi[4])
{
    lo[0] = lo[1] = lo[2] = lo[3] = 0;
    hi[0] = hi[1] = hi[2] = hi[3] = 0;
    for (int w = 0; w < 64; ++w) {
        const uint32_t v = row64[w];
        lo[w >> 4] |= (v & 3u) << (2 * (w & 15));
        if (bits == 3) {
            const int d = w >> 4, a = (w >> 3) & 1, e = w & 7;
            const int bit = 8 * ((e >> 2) + 2 * (e & 1)) + 2 * d + ((e & 3) >> 1);
            hi[a] |= ((v >> 2) & 1u) << bit;
        }
        if (bits == 4) hi[w >> 4] |= ((v >> 2) & 3u) << (2 * (w & 15));
    }
}

static void put32(uint8_t *p, uint32_t v) { p[0] = v & 255; p[1] = (v >> 8) & 255; p[2] = (v >> 16) & 255; p[3] = v >> 24; }
static uint32_t get32(const uint8_t *p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24); }

}  // namespace lcd

using namespace lcd;

extern "C" {

int lcd_version(void) { return LCD_VERSION; }
int lcd_layout_revision(void) { return LCD_LAYOUT_REVISION; }
const char *lcd_last_error_string(void) { return g_err; }

const char *lcd_status_string(lcd_status st)
{
    switch (st) {
    case LCD_OK: return "LCD_OK";
    case LCD_ERR_NULL: return "LCD_ERR_NULL";
    case LCD_ERR_BAD_BITS: return "LCD_ERR_BAD_BITS";
    case LCD_ERR_BAD_SHAPE: return "LCD_ERR_BAD_SHAPE";
    case LCD_ERR_BAD_M: return "LCD_ERR_BAD_M";
    case LCD_ERR_SIZE: return "LCD_ERR_SIZE";
    case LCD_ERR_INDEX_RANGE: return "LCD_ERR_INDEX_RANGE";
    case LCD_ERR_ALIGN: return "LCD_ERR_ALIGN";
    case LCD_ERR_HIP: return "LCD_ERR_HIP";
    case LCD_ERR_BAD_SCALE: return "LCD_ERR_BAD_SCALE";
    }
    return "LCD_ERR_UNKNOWN";
}

size_t lcd_packed_bytes(int N, int K, int bits)
{
    if (check_shape(N, K, bits) != LCD_OK) return 0;
    return (size_t)N * (size_t)K * (size_t)bits / 8;
}

size_t lcd_lut_bytes(int N, int bits)
{
    if (bits < 2 || bits > 4 || N <= 0 || N % kTileRows != 0) return 0;
    return (size_t)N * (bits == 2 ? 24 : bits == 3 ? 48 : 32);   // 4 bits: the byte-split tables only
}

size_t lcd_workspace_bytes(int M, int N, int K, int bits)
{
    if (check_shape(N, K, bits) != LCD_OK || M < 1) return 0;
    // the prefill path keeps the smoothed activations there; the decode path only the activation
    // codes of lcd_lut_gemv_q8 with M > 1 (M*K fp16 numbers, less than the prefill's M padded to 128)
    const GemmPlan m = plan_gemm(M, N, K, bits);
    return m.xs_bytes < 256 ? 256 : m.xs_bytes;
}

lcd_status lcd_pack_indices_host(const uint8_t *idx, int N, int K, int bits, void *packed, size_t packed_bytes)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (!idx) return fail(LCD_ERR_NULL, "idx is NULL");
    if (!packed) return fail(LCD_ERR_NULL, "packed is NULL");
    const size_t need = lcd_packed_bytes(N, K, bits);
    if (packed_bytes < need) return fail(LCD_ERR_SIZE, "packed_bytes=%zu < %zu", packed_bytes, need);
    const int lim = 1 << bits;
    for (size_t e = 0, n = (size_t)N * K; e < n; ++e)
        if (idx[e] >= lim) return fail(LCD_ERR_INDEX_RANGE, "idx[%zu]=%d >= %d", e, (int)idx[e], lim);
    uint8_t *out = static_cast<uint8_t *>(packed);
    const int kc = K / kTileCols;
    const size_t tb = tile_bytes(bits);
    for (int t = 0; t < N / kTileRows; ++t)
        for (int c = 0; c < kc; ++c) {
            uint8_t *tile = out + ((size_t)t * kc + c) * tb;
            for (int l = 0; l < 64; ++l) {
                const int q = l >> 4, i = l & 15;
                uint32_t lo[4], hi[4];
                lane_words(idx + (size_t)(t * kTileRows + i) * K + (size_t)c * kTileCols + q * kLaneCols, bits, lo, hi);
                for (int d = 0; d < 4; ++d) put32(tile + 16 * l + 4 * d, lo[d]);
                if (bits == 3) { put32(tile + 1024 + 8 * l, hi[0]); put32(tile + 1024 + 8 * l + 4, hi[1]); }
                if (bits == 4) for (int d = 0; d < 4; ++d) put32(tile + 1024 + 16 * l + 4 * d, hi[d]);
            }
        }
    return LCD_OK;
}

lcd_status lcd_unpack_indices_host(const void *packed, int N, int K, int bits, uint8_t *idx)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (!idx) return fail(LCD_ERR_NULL, "idx is NULL");
    if (!packed) return fail(LCD_ERR_NULL, "packed is NULL");
    const uint8_t *in = static_cast<const uint8_t *>(packed);
    const int kc = K / kTileCols;
    const size_t tb = tile_bytes(bits);
    for (int t = 0; t < N / kTileRows; ++t)
        for (int c = 0; c < kc; ++c) {
            const uint8_t *tile = in + ((size_t)t * kc + c) * tb;
            for (int l = 0; l < 64; ++l) {
                const int q = l >> 4, i = l & 15;
                uint8_t *row64 = idx + (size_t)(t * kTileRows + i) * K + (size_t)c * kTileCols + q * kLaneCols;
                uint32_t hi[2] = {0, 0};
                if (bits == 3) { hi[0] = get32(tile + 1024 + 8 * l); hi[1] = get32(tile + 1024 + 8 * l + 4); }
                for (int w = 0; w < 64; ++w) {
                    uint32_t v = (get32(tile + 16 * l + 4 * (w >> 4)) >> (2 * (w & 15))) & 3u;
                    if (bits == 3) {
                        const int d = w >> 4, a = (w >> 3) & 1, e = w & 7;
                        const int bit = 8 * ((e >> 2) + 2 * (e & 1)) + 2 * d + ((e & 3) >> 1);
                        v |= ((hi[a] >> bit) & 1u) << 2;
                    }
                    if (bits == 4) v |= ((get32(tile + 1024 + 16 * l + 4 * (w >> 4)) >> (2 * (w & 15))) & 3u) << 2;
                    row64[w] = (uint8_t)v;
                }
            }
        }
    return LCD_OK;
}

lcd_status lcd_pack_indices(const uint8_t *idx, int N, int K, int bits, void *packed, size_t packed_bytes, void *stream)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (lcd_status st = check_aligned(idx, "idx")) return st;
    if (lcd_status st = check_aligned(packed, "packed")) return st;
    const size_t need = lcd_packed_bytes(N, K, bits);
    if (packed_bytes < need) return fail(LCD_ERR_SIZE, "packed_bytes=%zu < %zu", packed_bytes, need);
    if (int e = launch_pack(idx, N, K, bits, packed, stream)) return fail(LCD_ERR_HIP, "pack launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_unpack_indices(const void *packed, int N, int K, int bits, uint8_t *idx, void *stream)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (lcd_status st = check_aligned(packed, "packed")) return st;
    if (lcd_status st = check_aligned(idx, "idx")) return st;
    if (int e = launch_unpack(packed, N, K, bits, idx, stream)) return fail(LCD_ERR_HIP, "unpack launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_build_lut(const uint16_t *codebook, int N, int bits, void *lut, size_t lut_bytes, void *stream)
{
    if (bits < 2 || bits > 4) return fail(LCD_ERR_BAD_BITS, "bits=%d: only 2, 3 and 4 are supported", bits);
    if (N <= 0 || N % kTileRows != 0) return fail(LCD_ERR_BAD_SHAPE, "N=%d must be a positive multiple of %d", N, kTileRows);
    if (lcd_status st = check_aligned(codebook, "codebook")) return st;
    if (lcd_status st = check_aligned(lut, "lut")) return st;
    const size_t need = lcd_lut_bytes(N, bits);
    if (lut_bytes < need) return fail(LCD_ERR_SIZE, "lut_bytes=%zu < %zu", lut_bytes, need);
    if (int e = launch_build_lut(codebook, N, bits, lut, stream)) return fail(LCD_ERR_HIP, "build_lut launch: %s", hip_error_name(e));
    return LCD_OK;
}

static lcd_status check_operands(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                                 int M, int N, int K, int bits)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (M < 1) return fail(LCD_ERR_BAD_M, "M=%d must be >= 1", M);
    if (lcd_status st = check_aligned(packed, "packed")) return st;
    if (lcd_status st = check_aligned(lut, "lut")) return st;
    if (lcd_status st = check_aligned(x, "x")) return st;
    if (lcd_status st = check_aligned(s, "s")) return st;
    if (lcd_status st = check_aligned(y, "y")) return st;
    return LCD_OK;
}

static lcd_status check_product(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                                int M, int N, int K, int bits, void *workspace, size_t workspace_bytes)
{
    if (lcd_status st = check_operands(packed, lut, x, s, y, M, N, K, bits)) return st;
    if (lcd_status st = check_aligned(workspace, "workspace")) return st;
    const size_t need = lcd_workspace_bytes(M, N, K, bits);
    if (workspace_bytes < need) return fail(LCD_ERR_SIZE, "workspace_bytes=%zu < %zu", workspace_bytes, need);
    return LCD_OK;
}

lcd_status lcd_lut_gemv(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                        int M, int N, int K, int bits, void *workspace, size_t workspace_bytes, void *stream)
{
    if (M > 16) return fail(LCD_ERR_BAD_M, "lcd_lut_gemv: M=%d > 16 (use lcd_lut_gemm)", M);
    if (lcd_status st = check_product(packed, lut, x, s, y, M, N, K, bits, workspace, workspace_bytes)) return st;
    if (int e = launch_gemv(packed, lut, x, s, y, M, N, K, bits, 0.0f, workspace, stream))
        return fail(LCD_ERR_HIP, "gemv launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_lut_gemv_noalloc(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                                int M, int N, int K, int bits, void *stream)
{
    if (M > 16) return fail(LCD_ERR_BAD_M, "lcd_lut_gemv_noalloc: M=%d > 16", M);
    if (lcd_status st = check_operands(packed, lut, x, s, y, M, N, K, bits)) return st;
    const size_t need = decode_codes_bytes(M, K);
    if (need > kStaticScratchBytes)
        return fail(LCD_ERR_SIZE, "lcd_lut_gemv_noalloc: M*K=%d*%d fp16 activations (%zu bytes) exceed the library's static scratch of %zu bytes",
                    M, K, need, kStaticScratchBytes);
    if (int e = launch_gemv_noalloc(packed, lut, x, s, y, M, N, K, bits, stream))
        return fail(LCD_ERR_HIP, "gemv launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_lut_gemv_q8(const void *packed, const void *lut, const uint16_t *x, const float *s, float s_q,
                           uint16_t *y, int M, int N, int K, int bits, void *workspace, size_t workspace_bytes, void *stream)
{
    if (M > 16) return fail(LCD_ERR_BAD_M, "lcd_lut_gemv_q8: M=%d > 16", M);
    if (!(s_q > 0.0f) || !(s_q < 3.0e38f)) return fail(LCD_ERR_BAD_SCALE, "s_q=%g must be positive and finite", (double)s_q);
    if (lcd_status st = check_product(packed, lut, x, s, y, M, N, K, bits, workspace, workspace_bytes)) return st;
    if (int e = launch_gemv(packed, lut, x, s, y, M, N, K, bits, s_q, workspace, stream))
        return fail(LCD_ERR_HIP, "gemv launch: %s", hip_error_name(e));
    return LCD_OK;
}

size_t lcd_workspace_bytes_grouped(const lcd_gemv_problem *problems, int count, int M, int bits)
{
    if (!problems || count < 1 || count > kMaxGroup || M < 1 || M > 16) return 0;
    size_t need = 256, codes = 0;   // the q8 variant keeps every layer's activation codes side by side
    for (int i = 0; i < count; ++i) {
        const size_t w = lcd_workspace_bytes(M, problems[i].N, problems[i].K, bits);
        if (w == 0) return 0;
        if (w > need) need = w;
        codes += decode_codes_bytes(M, problems[i].K);
    }
    return codes > need ? codes : need;
}

static lcd_status gemv_grouped(const lcd_gemv_problem *problems, const float *s_q, int count, int M, int bits,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    if (!problems) return fail(LCD_ERR_NULL, "problems is NULL");
    if (count < 1 || count > kMaxGroup) return fail(LCD_ERR_SIZE, "count=%d must be in 1..%d", count, kMaxGroup);
    if (M > 16) return fail(LCD_ERR_BAD_M, "grouped gemv: M=%d > 16", M);
    size_t codes = 0;
    for (int i = 0; i < count; ++i) {
        const lcd_gemv_problem &p = problems[i];
        if (lcd_status st = check_product(p.packed, p.lut, p.x, p.s, p.y, M, p.N, p.K, bits, workspace, workspace_bytes)) return st;
        codes += decode_codes_bytes(M, p.K);
        if (s_q && (!(s_q[i] > 0.0f) || !(s_q[i] < 3.0e38f)))
            return fail(LCD_ERR_BAD_SCALE, "s_q[%d]=%g must be positive and finite", i, (double)s_q[i]);
    }
    if (workspace_bytes < codes) return fail(LCD_ERR_SIZE, "workspace_bytes=%zu < %zu", workspace_bytes, codes);
    GroupItem items[kMaxGroup];
    for (int i = 0; i < count; ++i)
        items[i] = GroupItem{problems[i].packed, problems[i].lut, problems[i].x, problems[i].s, problems[i].y, problems[i].N, problems[i].K,
                             s_q ? s_q[i] : 0.0f};
    if (int e = launch_decode_group(items, count, M, bits, workspace, stream)) return fail(LCD_ERR_HIP, "grouped gemv launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_lut_gemv_grouped(const lcd_gemv_problem *problems, int count, int M, int bits,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return gemv_grouped(problems, nullptr, count, M, bits, workspace, workspace_bytes, stream);
}

lcd_status lcd_lut_gemv_q8_grouped(const lcd_gemv_problem *problems, const float *s_q, int count, int M, int bits,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!s_q) return fail(LCD_ERR_NULL, "s_q is NULL");
    return gemv_grouped(problems, s_q, count, M, bits, workspace, workspace_bytes, stream);
}

lcd_status lcd_lut_gemv_grouped_mixed(const lcd_gemv_problem *problems, const int *bits, int count, int M,
                                      void *workspace, size_t workspace_bytes, void *stream)
{
    if (!problems) return fail(LCD_ERR_NULL, "problems is NULL");
    if (!bits) return fail(LCD_ERR_NULL, "bits is NULL");
    if (count < 1 || count > kMaxGroup) return fail(LCD_ERR_SIZE, "count=%d must be in 1..%d", count, kMaxGroup);
    for (int i = 0; i < count; ++i)
        if (bits[i] < 2 || bits[i] > 4) return fail(LCD_ERR_BAD_BITS, "bits[%d]=%d: only 2, 3 and 4 are supported", i, bits[i]);
    // validate every layer before the first launch, then one launch per index width that occurs
    for (int pass = 0; pass < 2; ++pass)
        for (int b = 2; b <= 4; ++b) {
            lcd_gemv_problem sub[kMaxGroup];
            int n = 0;
            for (int i = 0; i < count; ++i)
                if (bits[i] == b) sub[n++] = problems[i];
            if (n == 0) continue;
            if (pass == 0) {
                if (M > 16) return fail(LCD_ERR_BAD_M, "grouped gemv: M=%d > 16", M);
                for (int i = 0; i < n; ++i)
                    if (lcd_status st = check_product(sub[i].packed, sub[i].lut, sub[i].x, sub[i].s, sub[i].y, M, sub[i].N, sub[i].K, b,
                                                      workspace, workspace_bytes)) return st;
            } else if (lcd_status st = gemv_grouped(sub, nullptr, n, M, b, workspace, workspace_bytes, stream)) {
                return st;
            }
        }
    return LCD_OK;
}

lcd_status lcd_lut_gemm(const void *packed, const void *lut, const uint16_t *x, const float *s, uint16_t *y,
                        int M, int N, int K, int bits, void *workspace, size_t workspace_bytes, void *stream)
{
    if (lcd_status st = check_product(packed, lut, x, s, y, M, N, K, bits, workspace, workspace_bytes)) return st;
    const GemmPlan plan = plan_gemm(M, N, K, bits);
    if (int e = launch_gemm(packed, lut, x, s, y, M, N, K, bits, 0.0f, workspace, plan, stream))
        return fail(LCD_ERR_HIP, "gemm launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_lut_gemm_q8(const void *packed, const void *lut, const uint16_t *x, const float *s, float s_q, uint16_t *y,
                           int M, int N, int K, int bits, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!(s_q > 0.0f) || !(s_q < 3.0e38f)) return fail(LCD_ERR_BAD_SCALE, "s_q=%g must be positive and finite", (double)s_q);
    if (lcd_status st = check_product(packed, lut, x, s, y, M, N, K, bits, workspace, workspace_bytes)) return st;
    const GemmPlan plan = plan_gemm(M, N, K, bits);
    if (int e = launch_gemm(packed, lut, x, s, y, M, N, K, bits, s_q, workspace, plan, stream))
        return fail(LCD_ERR_HIP, "gemm launch: %s", hip_error_name(e));
    return LCD_OK;
}

size_t lcd_workspace_bytes_gemm_grouped(const lcd_gemv_problem *problems, int count, int M, int bits)
{
    if (!problems || count < 1 || count > kMaxGroup || M < 1) return 0;
    size_t total = 0;
    for (int i = 0; i < count; ++i) {
        if (check_shape(problems[i].N, problems[i].K, bits) != LCD_OK) return 0;
        total += plan_gemm(M, problems[i].N, problems[i].K, bits).xs_bytes;
    }
    return total;
}

static lcd_status gemm_grouped(const lcd_gemv_problem *problems, const float *s_q, int count, int M, int bits,
                               void *workspace, size_t workspace_bytes, void *stream)
{
    if (!problems) return fail(LCD_ERR_NULL, "problems is NULL");
    if (count < 1 || count > kMaxGroup) return fail(LCD_ERR_SIZE, "count=%d must be in 1..%d", count, kMaxGroup);
    GroupItem items[kMaxGroup];
    size_t need = 0;
    for (int i = 0; i < count; ++i) {
        const lcd_gemv_problem &p = problems[i];
        // every layer's share of the workspace is checked below against the sum
        if (lcd_status st = check_product(p.packed, p.lut, p.x, p.s, p.y, M, p.N, p.K, bits, workspace, (size_t)-1)) return st;
        need += plan_gemm(M, p.N, p.K, bits).xs_bytes;
        if (s_q && (!(s_q[i] > 0.0f) || !(s_q[i] < 3.0e38f)))
            return fail(LCD_ERR_BAD_SCALE, "s_q[%d]=%g must be positive and finite", i, (double)s_q[i]);
        items[i] = GroupItem{p.packed, p.lut, p.x, p.s, p.y, p.N, p.K, s_q ? s_q[i] : 0.0f};
    }
    if (workspace_bytes < need) return fail(LCD_ERR_SIZE, "workspace_bytes=%zu < %zu", workspace_bytes, need);
    if (int e = launch_gemm_group(items, count, M, bits, workspace, stream))
        return fail(LCD_ERR_HIP, "grouped gemm launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_lut_gemm_grouped(const lcd_gemv_problem *problems, int count, int M, int bits,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    return gemm_grouped(problems, nullptr, count, M, bits, workspace, workspace_bytes, stream);
}

lcd_status lcd_lut_gemm_q8_grouped(const lcd_gemv_problem *problems, const float *s_q, int count, int M, int bits,
                                   void *workspace, size_t workspace_bytes, void *stream)
{
    if (!s_q) return fail(LCD_ERR_NULL, "s_q is NULL");
    return gemm_grouped(problems, s_q, count, M, bits, workspace, workspace_bytes, stream);
}

static lcd_status check_ncent(int ncent, int bits, int least)
{
    if (ncent < least || ncent > (1 << bits))
        return fail(LCD_ERR_SIZE, "ncent=%d must be in %d..%d for bits=%d", ncent, least, 1 << bits, bits);
    return LCD_OK;
}

lcd_status lcd_assign_indices(const uint16_t *w, const uint16_t *codebook, int ncent, int N, int K, int bits, uint8_t *idx, void *stream)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (lcd_status st = check_ncent(ncent, bits, 1)) return st;
    if (lcd_status st = check_aligned(w, "w")) return st;
    if (lcd_status st = check_aligned(codebook, "codebook")) return st;
    if (lcd_status st = check_aligned(idx, "idx")) return st;
    if (int e = launch_assign(w, codebook, ncent, N, K, bits, idx, stream)) return fail(LCD_ERR_HIP, "assign launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_cluster_counts(const uint8_t *idx, int N, int K, int bits, uint32_t *counts, void *stream)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (lcd_status st = check_aligned(idx, "idx")) return st;
    if (lcd_status st = check_aligned(counts, "counts")) return st;
    if (int e = launch_counts(idx, N, K, bits, counts, stream)) return fail(LCD_ERR_HIP, "counts launch: %s", hip_error_name(e));
    return LCD_OK;
}

lcd_status lcd_merge_closest(const uint16_t *codebook, const uint32_t *counts, const uint8_t *idx, int ncent, int N, int K, int bits,
                             uint16_t *codebook_out, uint8_t *idx_out, uint8_t *merged, void *stream)
{
    if (lcd_status st = check_shape(N, K, bits)) return st;
    if (lcd_status st = check_ncent(ncent, bits, 2)) return st;
    if (lcd_status st = check_aligned(codebook, "codebook")) return st;
    if (lcd_status st = check_aligned(counts, "counts")) return st;
    if (lcd_status st = check_aligned(idx, "idx")) return st;
    if (lcd_status st = check_aligned(codebook_out, "codebook_out")) return st;
    if (lcd_status st = check_aligned(idx_out, "idx_out")) return st;
    if (lcd_status st = check_aligned(merged, "merged")) return st;
    if (codebook_out == codebook) return fail(LCD_ERR_SIZE, "codebook_out must not be the input codebook");
    if (int e = launch_merge(codebook, counts, idx, ncent, N, K, bits, codebook_out, idx_out, merged, stream))
        return fail(LCD_ERR_HIP, "merge launch: %s", hip_error_name(e));
    return LCD_OK;
}

}  // extern "C"
