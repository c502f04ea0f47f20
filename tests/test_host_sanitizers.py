"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, gcc).

The C oracle and the host side of the C ABI (argument validation, size arithmetic, the host twins of
the index packer) are built with -fsanitize=address,undefined together with a small C driver and run:
packer round trips at 2, 3 and 4 bits with buffers of exactly the stated sizes (so one byte too far is
a report), every error path of the host packer, the validation of the device entry points (which must
fail before any launch), and one small oracle product checked against a loop written out in the driver.
The GPU launchers are replaced by stubs that must never be reached.
"""
import os
import shutil
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
CSRC = ROOT / "paper_2506_12038_amd" / "csrc"

STUBS = r"""
// Stand-ins for the GPU launchers: host-only build.  Reaching one means validation let a call through.
#include <cstdio>
#include <cstdlib>
#include "lcd_internal.h"
namespace lcd {
static int reached(const char *what) { std::fprintf(stderr, "launcher reached: %s\n", what); std::abort(); return 1; }
int launch_pack(const uint8_t *, int, int, int, void *, void *) { return reached("pack"); }
int launch_unpack(const void *, int, int, int, uint8_t *, void *) { return reached("unpack"); }
int launch_build_lut(const uint16_t *, int, int, void *, void *) { return reached("build_lut"); }
int launch_gemv(const void *, const void *, const uint16_t *, const float *, uint16_t *, int, int, int, int, float, void *, void *) { return reached("gemv"); }
int launch_gemv_noalloc(const void *, const void *, const uint16_t *, const float *, uint16_t *, int, int, int, int, void *) { return reached("gemv_noalloc"); }
int launch_gemm(const void *, const void *, const uint16_t *, const float *, uint16_t *, int, int, int, int, float, void *, const GemmPlan &, void *) { return reached("gemm"); }
int launch_assign(const uint16_t *, const uint16_t *, int, int, int, int, uint8_t *, void *) { return reached("assign"); }
int launch_counts(const uint8_t *, int, int, int, uint32_t *, void *) { return reached("counts"); }
int launch_merge(const uint16_t *, const uint32_t *, const uint8_t *, int, int, int, int, uint16_t *, uint8_t *, uint8_t *, void *) { return reached("merge"); }
int launch_decode_group(const GroupItem *, int, int, int, void *, void *, bool) { return reached("decode_group"); }
int launch_gemm_group(const GroupItem *, int, int, int, void *, void *) { return reached("gemm_group"); }
const char *hip_error_name(int) { return "stub"; }
}
"""

DRIVER = r"""
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "lcd.h"

int oracle_lut_matmul(const uint16_t *, const uint8_t *, const uint16_t *, const float *, int, int, int, int, double *);
int oracle_bucket_matmul(const uint16_t *, const uint8_t *, const uint16_t *, const float *, int, int, int, int, double *);
int oracle_dequant(const uint16_t *, const uint8_t *, int, int, int, double *);
void oracle_smooth(const uint16_t *, const float *, int, int, double *);
void oracle_input_transform(const uint16_t *, const float *, double, int, int, int, int32_t *);
void oracle_input_transform_f32(const uint16_t *, const float *, float, int, int, int, int32_t *);
double oracle_half_to_double(uint16_t);

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "%s:%d: %s\n", __FILE__, __LINE__, #c); return 1; } } while (0)

static unsigned rnd_state = 12345u;
static unsigned rnd(void) { rnd_state = rnd_state * 1664525u + 1013904223u; return rnd_state >> 8; }

int main(void)
{
    /* packer round trips: every buffer has exactly the size the interface states */
    for (int bits = 2; bits <= 4; ++bits) {
        const int shapes[3][2] = {{16, 256}, {48, 768}, {32, 1280}};
        for (int sh = 0; sh < 3; ++sh) {
            const int N = shapes[sh][0], K = shapes[sh][1];
            const size_t nb = lcd_packed_bytes(N, K, bits);
            CHECK(nb == (size_t)N * K * bits / 8);
            uint8_t *idx = malloc((size_t)N * K), *back = malloc((size_t)N * K), *packed = malloc(nb);
            CHECK(idx && back && packed);
            for (size_t i = 0; i < (size_t)N * K; ++i) idx[i] = (uint8_t)(rnd() % (1u << bits));
            CHECK(lcd_pack_indices_host(idx, N, K, bits, packed, nb) == LCD_OK);
            memset(back, 0xEE, (size_t)N * K);
            CHECK(lcd_unpack_indices_host(packed, N, K, bits, back) == LCD_OK);
            CHECK(memcmp(idx, back, (size_t)N * K) == 0);
            /* error paths of the host packer: nothing may be written */
            memset(packed, 0x5A, nb);
            CHECK(lcd_pack_indices_host(idx, N, K, bits, packed, nb - 1) == LCD_ERR_SIZE);
            idx[(size_t)N * K - 1] = (uint8_t)(1u << bits);
            CHECK(lcd_pack_indices_host(idx, N, K, bits, packed, nb) == LCD_ERR_INDEX_RANGE);
            for (size_t i = 0; i < nb; ++i) CHECK(packed[i] == 0x5A);
            CHECK(strlen(lcd_last_error_string()) > 0);
            CHECK(lcd_pack_indices_host(NULL, N, K, bits, packed, nb) == LCD_ERR_NULL);
            CHECK(lcd_pack_indices_host(idx, N, K, bits, NULL, nb) == LCD_ERR_NULL);
            CHECK(lcd_pack_indices_host(idx, N - 1, K, bits, packed, nb) == LCD_ERR_BAD_SHAPE);
            CHECK(lcd_pack_indices_host(idx, N, K - 1, bits, packed, nb) == LCD_ERR_BAD_SHAPE);
            CHECK(lcd_unpack_indices_host(NULL, N, K, bits, back) == LCD_ERR_NULL);
            free(idx); free(back); free(packed);
        }
    }
    CHECK(lcd_packed_bytes(16, 256, 5) == 0 && lcd_packed_bytes(0, 256, 2) == 0 && lcd_packed_bytes(16, -256, 2) == 0);
    CHECK(lcd_packed_bytes(1 << 20, 1 << 20, 4) == 0);                    /* 4 GiB and more is refused, no overflow */
    CHECK(lcd_lut_bytes(16, 2) == 16 * 24 && lcd_lut_bytes(16, 3) == 16 * 48 && lcd_lut_bytes(16, 4) == 16 * 32 && lcd_lut_bytes(15, 2) == 0);
    CHECK(lcd_workspace_bytes(2048, 4096, 4096, 3) >= (size_t)2048 * 4096 * 2 && lcd_workspace_bytes(0, 16, 256, 2) == 0);
    for (int st = 0; st <= 10; ++st) CHECK(strlen(lcd_status_string((lcd_status)st)) > 4);

    /* device entry points: validation fails on the host, before any launch (the stubs abort) */
    void *a = (void *)(uintptr_t)0x1000, *odd = (void *)(uintptr_t)0x1004;
    CHECK(lcd_pack_indices(NULL, 16, 256, 2, a, 1024, NULL) == LCD_ERR_NULL);
    CHECK(lcd_pack_indices(a, 16, 256, 2, a, 1000, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_unpack_indices(a, 16, 250, 2, a, NULL) == LCD_ERR_BAD_SHAPE);
    CHECK(lcd_build_lut(a, 16, 2, a, 10, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_lut_gemv(a, a, a, a, a, 17, 16, 256, 2, a, 1 << 20, NULL) == LCD_ERR_BAD_M);
    CHECK(lcd_lut_gemv(a, a, a, odd, a, 1, 16, 256, 2, a, 1 << 20, NULL) == LCD_ERR_ALIGN);
    CHECK(lcd_lut_gemv(a, a, a, a, a, 1, 16, 256, 2, a, 0, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_lut_gemv_noalloc(a, a, a, a, a, 16, 16, 33024, 2, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_lut_gemv_q8(a, a, a, a, 0.0f, a, 1, 16, 256, 2, a, 1 << 20, NULL) == LCD_ERR_BAD_SCALE);
    CHECK(lcd_lut_gemm(a, a, NULL, a, a, 64, 16, 256, 3, a, 1 << 20, NULL) == LCD_ERR_NULL);
    CHECK(lcd_lut_gemm_q8(a, a, a, a, -0.5f, a, 64, 16, 256, 3, a, 1 << 20, NULL) == LCD_ERR_BAD_SCALE);
    CHECK(lcd_lut_gemm_q8(a, a, a, a, 0.5f, a, 64, 16, 256, 3, a, 16, NULL) == LCD_ERR_SIZE);
    lcd_gemv_problem pr[17];
    for (int i = 0; i < 17; ++i) { pr[i].packed = a; pr[i].lut = a; pr[i].x = a; pr[i].s = a; pr[i].y = a; pr[i].N = 16 * (i + 1); pr[i].K = 256 * (i + 1); }
    CHECK(lcd_workspace_bytes_grouped(pr, 16, 16, 2) >= 16 * 256 * 136 * 2);
    CHECK(lcd_lut_gemv_grouped(pr, 17, 1, 2, a, 1 << 20, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_lut_gemv_grouped(pr, 16, 17, 2, a, 1 << 20, NULL) == LCD_ERR_BAD_M);
    CHECK(lcd_lut_gemv_grouped(pr, 16, 16, 2, a, 4096, NULL) == LCD_ERR_SIZE);
    pr[15].y = odd;
    CHECK(lcd_lut_gemv_grouped(pr, 16, 1, 2, a, 1 << 20, NULL) == LCD_ERR_ALIGN);
    CHECK(lcd_lut_gemm_grouped(pr, 16, 64, 3, a, 1 << 20, NULL) == LCD_ERR_ALIGN);
    pr[15].y = a;
    CHECK(lcd_lut_gemm_grouped(pr, 16, 64, 3, a, 1024, NULL) == LCD_ERR_SIZE);
    int widths[16]; for (int i = 0; i < 16; ++i) widths[i] = 2 + i % 3;
    widths[7] = 5;
    CHECK(lcd_lut_gemv_grouped_mixed(pr, widths, 16, 1, a, 1 << 20, NULL) == LCD_ERR_BAD_BITS);
    float sq[16]; for (int i = 0; i < 16; ++i) sq[i] = 0.1f;
    sq[15] = -1.0f;
    CHECK(lcd_lut_gemv_q8_grouped(pr, sq, 16, 1, 2, a, 1 << 20, NULL) == LCD_ERR_BAD_SCALE);
    CHECK(lcd_lut_gemm_q8_grouped(pr, sq, 16, 64, 2, a, 1 << 30, NULL) == LCD_ERR_BAD_SCALE);
    CHECK(lcd_lut_gemm_q8_grouped(pr, NULL, 16, 64, 2, a, 1 << 30, NULL) == LCD_ERR_NULL);
    CHECK(lcd_assign_indices(a, a, 5, 16, 256, 2, a, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_merge_closest(a, a, a, 1, 16, 256, 2, a, a, a, NULL) == LCD_ERR_SIZE);
    CHECK(lcd_cluster_counts(a, 16, 256, 2, odd, NULL) == LCD_ERR_ALIGN);

    /* one small oracle product against a loop written out here (fp16 inputs built from integers) */
    enum { M = 3, N = 5, K = 37, BITS = 3 };
    uint16_t cb[N * 8], x[M * K];
    uint8_t idx[N * K];
    float s[K];
    double Y[M * N], Yb[M * N], W[N * K], xs[M * K];
    int32_t q[M * K], q32[M * K];
    for (int i = 0; i < N * 8; ++i) cb[i] = (uint16_t)(0x2000 + rnd() % 0x1000 + ((rnd() & 1) << 15));   /* normal numbers around 2^-7 */
    for (int i = 0; i < M * K; ++i) x[i] = (uint16_t)(0x3800 + rnd() % 0x1000 + ((rnd() & 1) << 15));
    for (int i = 0; i < N * K; ++i) idx[i] = (uint8_t)(rnd() % 8);
    for (int k = 0; k < K; ++k) s[k] = 0.5f + (float)(rnd() % 1000) / 500.0f;
    CHECK(oracle_lut_matmul(cb, idx, x, s, M, N, K, BITS, Y) == 0);
    CHECK(oracle_bucket_matmul(cb, idx, x, s, M, N, K, BITS, Yb) == 0);
    CHECK(oracle_dequant(cb, idx, N, K, BITS, W) == 0);
    oracle_smooth(x, s, M, K, xs);
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0, mag = 0.0;
            for (int k = 0; k < K; ++k) { acc += xs[m * K + k] * W[n * K + k]; mag += fabs(xs[m * K + k] * W[n * K + k]); }
            CHECK(fabs(acc - Y[m * N + n]) <= mag * 1e-14);
            CHECK(fabs(acc - Yb[m * N + n]) <= mag * 1e-14);
        }
    idx[7] = 8;
    CHECK(oracle_lut_matmul(cb, idx, x, s, M, N, K, BITS, Y) == 1);      /* out-of-range index reported, no wild read */
    oracle_input_transform(x, s, 0.01, 8, M, K, q);
    oracle_input_transform_f32(x, s, 0.01f, 8, M, K, q32);
    for (int i = 0; i < M * K; ++i) CHECK(q[i] >= -128 && q[i] <= 127 && abs(q[i] - q32[i]) <= 1);
    CHECK(oracle_half_to_double(0x3c00) == 1.0 && oracle_half_to_double(0xfbff) == -65504.0);
    puts("sanitized host code: ok");
    return 0;
}
"""


@pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="gcc/g++ not found")
def test_host_side_and_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    inc = [f"-I{ROOT / 'include'}", f"-I{CSRC}"]
    (tmp_path / "stubs.cpp").write_text(STUBS)
    (tmp_path / "driver.c").write_text(DRIVER)
    objs = []
    for compiler, src, extra in (("g++", CSRC / "lcd_host.cpp", ["-std=c++17"]), ("g++", tmp_path / "stubs.cpp", ["-std=c++17"]),
                                 ("gcc", ROOT / "oracle" / "lcd_oracle.c", ["-std=c11", "-fno-fast-math"]),
                                 ("gcc", tmp_path / "driver.c", ["-std=c11", "-D_DEFAULT_SOURCE"])):
        obj = tmp_path / (Path(src).stem + ".o")
        subprocess.check_call([compiler, *san, *extra, *inc, "-c", str(src), "-o", str(obj)])
        objs.append(str(obj))
    exe = tmp_path / "sanitized"
    # the sanitizer runtime linked statically: its start-up check does not depend on what else is preloaded
    subprocess.check_call(["g++", *san, "-static-libasan", *objs, "-o", str(exe), "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([str(exe)], capture_output=True, text=True, env=env, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitized host code: ok" in run.stdout
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr
