"""CPU-only tests of the C-ABI library: exports, size arithmetic, host packer, error paths."""
import ctypes
import re
from pathlib import Path

import numpy as np
import pytest

import paper_2506_12038_amd as lcd
from oracle.pack_ref import pack_ref, unpack_ref

ROOT = Path(__file__).resolve().parent.parent


def declared_functions():
    text = (ROOT / "include" / "lcd.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lcd_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = lcd.load_library()
    names = declared_functions()
    assert "lcd_lut_gemv" in names and "lcd_pack_indices" in names and len(names) >= 14
    for name in names:
        assert hasattr(lib, name), f"{name} declared in lcd.h but not exported"
    assert set(lcd.EXPORTS) == set(names)
    assert lcd.lcd_version() >= 100 and lcd.lcd_layout_revision() == 1


def test_size_functions():
    assert lcd.lcd_packed_bytes(4096, 4096, 2) == 4194304
    assert lcd.lcd_packed_bytes(4096, 4096, 3) == 6291456
    assert lcd.lcd_packed_bytes(11008, 4096, 3) == 16908288
    assert lcd.lcd_packed_bytes(28672, 8192, 2) == 58720256
    assert lcd.lcd_packed_bytes(4096, 4096, 4) == 8388608
    assert lcd.lcd_packed_bytes(4096, 4096, 5) == 0 and lcd.lcd_packed_bytes(4096, 4096, 1) == 0
    assert lcd.lcd_packed_bytes(4100, 4096, 2) == 0 and lcd.lcd_packed_bytes(4096, 4100, 2) == 0
    assert lcd.lcd_lut_bytes(4096, 2) == 4096 * 24 and lcd.lcd_lut_bytes(4096, 3) == 4096 * 48 and lcd.lcd_lut_bytes(4096, 4) == 4096 * 32
    for M, N, K, bits in [(1, 4096, 4096, 2), (16, 11008, 4096, 2), (2048, 4096, 11008, 3), (8, 8192, 28672, 2)]:
        w = lcd.lcd_workspace_bytes(M, N, K, bits)
        assert w >= 256 and w % 256 == 0
    assert lcd.lcd_workspace_bytes(0, 4096, 4096, 2) == 0


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (32, 1024)])
def test_host_packer_matches_layout_definition(bits, shape):
    N, K = shape
    idx = np.random.default_rng(10 * bits + N).integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    packed = lcd.lcd_pack_indices_host(idx, bits)
    assert packed.size == N * K * bits // 8
    assert np.array_equal(packed, pack_ref(idx, bits))
    assert np.array_equal(lcd.lcd_unpack_indices_host(packed, N, K, bits), idx)
    assert np.array_equal(unpack_ref(packed, N, K, bits), idx)


def test_golden_bytes_hand_worked():
    # One 16x256 tile, all zero except four entries; byte positions worked by hand from the
    # layout text in lcd.h:
    #  (n=0,k=0)=3   -> lane 0, w=0: bits [1:0] of tile byte 0            -> byte 0 = 0x03
    #  (n=1,k=5)=2   -> lane 1, w=5: bits [11:10] of the word at byte 16  -> byte 17 = 0x08
    #  (n=2,k=64)=1  -> lane 16+2, w=0: word at byte 288                  -> byte 288 = 0x01
    #  (n=15,k=255)=3-> lane 48+15=63, w=63: bits [127:126] at byte 1008  -> byte 1023 = 0xC0
    idx = np.zeros((16, 256), dtype=np.uint8)
    idx[0, 0] = 3; idx[1, 5] = 2; idx[2, 64] = 1; idx[15, 255] = 3
    p = lcd.lcd_pack_indices_host(idx, 2)
    expect = np.zeros(1024, dtype=np.uint8)
    expect[0] = 0x03; expect[17] = 0x08; expect[288] = 0x01; expect[1023] = 0xC0
    assert np.array_equal(p, expect)
    assert np.array_equal(pack_ref(idx, 2), expect)          # the oracle's layout packer against the same hand-worked bytes
    # 3-bit: same low fields plus the third-bit plane.
    #  (n=0,k=0)=7:  w=0 -> d=0,a=0,e=0 -> word 0 of lane 0, bit 0        -> byte 1024 = 0x01
    #  (n=1,k=5)=6:  w=5 -> d=0,a=0,e=5 -> bit 8*(1+2)+0+0 = 24           -> byte 1024+8+3 = 0x01
    #  (n=2,k=64+27)=4: lane 18, w=27 -> d=1,a=1,e=3 -> word 1, bit 8*(0+2)+2+1 = 19 -> byte 1024+144+4+2 = 0x08
    idx3 = np.zeros((16, 256), dtype=np.uint8)
    idx3[0, 0] = 7; idx3[1, 5] = 6; idx3[2, 91] = 4
    p3 = lcd.lcd_pack_indices_host(idx3, 3)
    e3 = np.zeros(1536, dtype=np.uint8)
    e3[0] = 0x03; e3[17] = 0x08
    e3[1024] = 0x01; e3[1024 + 8 + 3] = 0x01; e3[1024 + 144 + 4 + 2] = 0x08
    assert np.array_equal(p3, e3)
    assert np.array_equal(pack_ref(idx3, 3), e3)
    # 4-bit: the low fields as before, index bits 3:2 in the same arrangement 1024 bytes further on.
    #  (n=0,k=0)=15    -> low byte 0 = 0x03, high field: bits [1:0] of tile byte 1024      -> 0x03
    #  (n=1,k=5)=9     -> low = 1: byte 17 = 0x04; high = 2: bits [11:10] at byte 1024+16  -> byte 1041 = 0x08
    #  (n=2,k=64)=4    -> low = 0; high = 1: lane 18, word at byte 1024+288                -> byte 1312 = 0x01
    #  (n=15,k=255)=14 -> low = 2: byte 1023 = 0x80; high = 3: byte 2047 = 0xC0
    idx4 = np.zeros((16, 256), dtype=np.uint8)
    idx4[0, 0] = 15; idx4[1, 5] = 9; idx4[2, 64] = 4; idx4[15, 255] = 14
    p4 = lcd.lcd_pack_indices_host(idx4, 4)
    e4 = np.zeros(2048, dtype=np.uint8)
    e4[0] = 0x03; e4[17] = 0x04; e4[1023] = 0x80
    e4[1024] = 0x03; e4[1041] = 0x08; e4[1312] = 0x01; e4[2047] = 0xC0
    assert np.array_equal(p4, e4)
    assert np.array_equal(pack_ref(idx4, 4), e4)


def test_host_packer_rejects_out_of_range_and_bad_shapes():
    idx = np.zeros((16, 256), dtype=np.uint8)
    idx[3, 7] = 4
    with pytest.raises(lcd.LcdError) as ei:
        lcd.lcd_pack_indices_host(idx, 2)
    assert ei.value.name == "LCD_ERR_INDEX_RANGE"
    lcd.lcd_pack_indices_host(idx, 3)  # 4 is fine for 3 bits
    lib = lcd.load_library()
    buf = np.zeros(4096, dtype=np.uint8)
    ok_idx = np.zeros((16, 256), dtype=np.uint8)
    ip, bp = ok_idx.ctypes.data_as(ctypes.c_void_p), buf.ctypes.data_as(ctypes.c_void_p)
    assert lib.lcd_status_string(lib.lcd_pack_indices_host(ip, 16, 256, 5, bp, 4096)) == b"LCD_ERR_BAD_BITS"
    assert lib.lcd_status_string(lib.lcd_pack_indices_host(ip, 15, 256, 2, bp, 4096)) == b"LCD_ERR_BAD_SHAPE"
    assert lib.lcd_status_string(lib.lcd_pack_indices_host(ip, 16, 128, 2, bp, 4096)) == b"LCD_ERR_BAD_SHAPE"
    assert lib.lcd_status_string(lib.lcd_pack_indices_host(ip, 16, 256, 2, bp, 100)) == b"LCD_ERR_SIZE"
    assert lib.lcd_status_string(lib.lcd_pack_indices_host(None, 16, 256, 2, bp, 4096)) == b"LCD_ERR_NULL"
    assert b"packed_bytes" in lib.lcd_last_error_string() or b"NULL" in lib.lcd_last_error_string()


def test_device_entry_points_validate_before_launch():
    # Host-side validation fails before any HIP call, so these run without a GPU.
    lib = lcd.load_library()
    a = ctypes.c_void_p(0x1000)       # fake, aligned, never dereferenced: validation fails first
    odd = ctypes.c_void_p(0x1004)
    st = lambda code: lib.lcd_status_string(code)
    assert st(lib.lcd_pack_indices(None, 16, 256, 2, a, 1024, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_pack_indices(odd, 16, 256, 2, a, 1024, None)) == b"LCD_ERR_ALIGN"
    assert st(lib.lcd_pack_indices(a, 16, 256, 2, a, 1000, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_unpack_indices(a, 16, 250, 2, a, None)) == b"LCD_ERR_BAD_SHAPE"
    assert st(lib.lcd_build_lut(a, 16, 5, a, 4096, None)) == b"LCD_ERR_BAD_BITS"
    assert st(lib.lcd_build_lut(a, 16, 2, a, 10, None)) == b"LCD_ERR_SIZE"
    big = 1 << 30
    assert st(lib.lcd_lut_gemv(a, a, a, a, a, 17, 16, 256, 2, a, big, None)) == b"LCD_ERR_BAD_M"
    assert st(lib.lcd_lut_gemv(a, a, a, a, a, 0, 16, 256, 2, a, big, None)) == b"LCD_ERR_BAD_M"
    assert st(lib.lcd_lut_gemv(a, a, a, a, a, 1, 16, 256, 2, a, 0, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_lut_gemv(a, a, a, odd, a, 1, 16, 256, 2, a, big, None)) == b"LCD_ERR_ALIGN"
    lib.lcd_lut_gemv_q8.argtypes = [ctypes.c_void_p] * 4 + [ctypes.c_float, ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert st(lib.lcd_lut_gemv_q8(a, a, a, a, 0.0, a, 1, 16, 256, 2, a, big, None)) == b"LCD_ERR_BAD_SCALE"
    assert st(lib.lcd_lut_gemv_q8(a, a, a, a, float("nan"), a, 1, 16, 256, 2, a, big, None)) == b"LCD_ERR_BAD_SCALE"
    assert st(lib.lcd_lut_gemv_q8(a, a, a, a, -1.0, a, 1, 16, 256, 2, a, big, None)) == b"LCD_ERR_BAD_SCALE"
    assert st(lib.lcd_lut_gemv_q8(a, a, a, a, 0.5, a, 17, 16, 256, 2, a, big, None)) == b"LCD_ERR_BAD_M"
    assert st(lib.lcd_lut_gemv_q8(a, None, a, a, 0.5, a, 1, 16, 256, 2, a, big, None)) == b"LCD_ERR_NULL"
    # the allocation-free variant: its static scratch holds 16 x 32768 fp16 activations
    assert st(lib.lcd_lut_gemv_noalloc(a, a, a, a, a, 17, 16, 256, 2, None)) == b"LCD_ERR_BAD_M"
    assert st(lib.lcd_lut_gemv_noalloc(a, a, a, a, a, 16, 16, 33024, 2, None)) == b"LCD_ERR_SIZE"
    assert b"static scratch" in lib.lcd_last_error_string()
    assert st(lib.lcd_lut_gemv_noalloc(a, a, a, a, a, 9, 16, 65536, 3, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_lut_gemv_noalloc(a, a, odd, a, a, 2, 16, 256, 2, None)) == b"LCD_ERR_ALIGN"
    assert st(lib.lcd_lut_gemv_noalloc(a, a, a, a, None, 2, 16, 256, 2, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_lut_gemm(a, a, None, a, a, 64, 16, 256, 3, a, big, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_lut_gemm(a, a, a, a, a, 64, 16, 256, 1, a, big, None)) == b"LCD_ERR_BAD_BITS"


def test_grouped_entry_point_validates_on_host():
    from paper_2506_12038_amd.binding import _Problem
    lib = lcd.load_library()
    a = 0x1000
    arr = (_Problem * 2)(_Problem(a, a, a, a, a, 16, 256), _Problem(a, a, a, a, a, 32, 512))
    st = lambda code: lib.lcd_status_string(code)
    big = 1 << 30
    assert lib.lcd_workspace_bytes_grouped(arr, 2, 1, 2) >= 256
    assert lib.lcd_workspace_bytes_grouped(arr, 0, 1, 2) == 0
    assert lib.lcd_workspace_bytes_grouped(arr, 2, 17, 2) == 0
    assert st(lib.lcd_lut_gemv_grouped(None, 2, 1, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_lut_gemv_grouped(arr, 17, 1, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_lut_gemv_grouped(arr, 2, 20, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_M"
    assert st(lib.lcd_lut_gemv_grouped(arr, 2, 1, 5, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_BITS"
    arr[1].K = 500
    assert st(lib.lcd_lut_gemv_grouped(arr, 2, 1, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_SHAPE"
    arr[1].K = 512
    arr[1].y = 0x1002
    assert st(lib.lcd_lut_gemv_grouped(arr, 2, 1, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_ALIGN"
    arr[1].y = a
    # the quantised variant: one positive finite step per layer, in a host array
    sq = (ctypes.c_float * 2)(0.05, 0.0)
    assert st(lib.lcd_lut_gemv_q8_grouped(arr, None, 2, 1, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_lut_gemv_q8_grouped(arr, sq, 2, 1, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_SCALE"
    sq[1] = float("inf")
    assert st(lib.lcd_lut_gemv_q8_grouped(arr, sq, 2, 4, 2, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_SCALE"
    sq[1] = 0.25
    # several tokens: the workspace holds every layer's activation codes side by side
    need = lib.lcd_workspace_bytes_grouped(arr, 2, 16, 2)
    assert need >= 16 * (256 + 512) * 2
    assert st(lib.lcd_lut_gemv_q8_grouped(arr, sq, 2, 16, 2, ctypes.c_void_p(a), 16 * 512 * 2, None)) == b"LCD_ERR_SIZE"
    # mixed index widths: a host array of widths, validated like everything else
    widths = (ctypes.c_int * 2)(2, 5)
    assert st(lib.lcd_lut_gemv_grouped_mixed(arr, None, 2, 1, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_lut_gemv_grouped_mixed(arr, widths, 2, 1, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_BITS"
    widths[1] = 4
    assert st(lib.lcd_lut_gemv_grouped_mixed(arr, widths, 2, 17, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_M"
    arr[0].K = 100
    assert st(lib.lcd_lut_gemv_grouped_mixed(arr, widths, 2, 1, ctypes.c_void_p(a), big, None)) == b"LCD_ERR_BAD_SHAPE"
    arr[0].K = 256
    assert st(lib.lcd_lut_gemv_grouped_mixed(arr, widths, 2, 4, ctypes.c_void_p(a), 256, None)) == b"LCD_ERR_SIZE"


def test_grouped_prefill_entry_point_validates_on_host():
    from paper_2506_12038_amd.binding import _Problem
    lib = lcd.load_library()
    a = 0x1000
    arr = (_Problem * 2)(_Problem(a, a, a, a, a, 16, 256), _Problem(a, a, a, a, a, 32, 512))
    st = lambda code: lib.lcd_status_string(code)
    # the workspace is the sum of the layers' own: smoothed activations side by side
    need = lib.lcd_workspace_bytes_gemm_grouped(arr, 2, 200, 3)
    assert need == lcd.lcd_workspace_bytes(200, 16, 256, 3) + lcd.lcd_workspace_bytes(200, 32, 512, 3)
    assert lib.lcd_workspace_bytes_gemm_grouped(arr, 0, 200, 3) == 0
    assert lib.lcd_workspace_bytes_gemm_grouped(arr, 17, 200, 3) == 0
    assert lib.lcd_workspace_bytes_gemm_grouped(arr, 2, 0, 3) == 0
    assert lib.lcd_workspace_bytes_gemm_grouped(arr, 2, 200, 5) == 0
    assert st(lib.lcd_lut_gemm_grouped(None, 2, 200, 3, ctypes.c_void_p(a), need, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_lut_gemm_grouped(arr, 0, 200, 3, ctypes.c_void_p(a), need, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_lut_gemm_grouped(arr, 2, 0, 3, ctypes.c_void_p(a), need, None)) == b"LCD_ERR_BAD_M"
    assert st(lib.lcd_lut_gemm_grouped(arr, 2, 200, 1, ctypes.c_void_p(a), need, None)) == b"LCD_ERR_BAD_BITS"
    assert st(lib.lcd_lut_gemm_grouped(arr, 2, 200, 3, ctypes.c_void_p(a), need - 256, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_lut_gemm_grouped(arr, 2, 200, 3, None, need, None)) == b"LCD_ERR_NULL"
    arr[1].N = 40
    assert st(lib.lcd_lut_gemm_grouped(arr, 2, 200, 3, ctypes.c_void_p(a), need, None)) == b"LCD_ERR_BAD_SHAPE"
    arr[1].N = 32
    arr[0].x = 0x1008
    assert st(lib.lcd_lut_gemm_grouped(arr, 2, 200, 3, ctypes.c_void_p(a), need, None)) == b"LCD_ERR_ALIGN"


def test_clustering_entry_points_validate_on_host():
    lib = lcd.load_library()
    a = ctypes.c_void_p(0x1000)
    odd = ctypes.c_void_p(0x1008)
    st = lambda code: lib.lcd_status_string(code)
    assert st(lib.lcd_assign_indices(None, a, 4, 16, 256, 2, a, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_assign_indices(a, odd, 4, 16, 256, 2, a, None)) == b"LCD_ERR_ALIGN"
    assert st(lib.lcd_assign_indices(a, a, 5, 16, 256, 2, a, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_assign_indices(a, a, 0, 16, 256, 2, a, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_assign_indices(a, a, 4, 16, 200, 2, a, None)) == b"LCD_ERR_BAD_SHAPE"
    assert st(lib.lcd_assign_indices(a, a, 4, 16, 256, 6, a, None)) == b"LCD_ERR_BAD_BITS"
    assert st(lib.lcd_cluster_counts(a, 16, 256, 3, None, None)) == b"LCD_ERR_NULL"
    assert st(lib.lcd_cluster_counts(a, 17, 256, 3, a, None)) == b"LCD_ERR_BAD_SHAPE"
    assert st(lib.lcd_merge_closest(a, a, a, 1, 16, 256, 3, ctypes.c_void_p(0x2000), a, a, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_merge_closest(a, a, a, 9, 16, 256, 3, ctypes.c_void_p(0x2000), a, a, None)) == b"LCD_ERR_SIZE"
    assert st(lib.lcd_merge_closest(a, a, a, 8, 16, 256, 3, a, a, a, None)) == b"LCD_ERR_SIZE"      # output over the input codebook
    assert st(lib.lcd_merge_closest(a, a, a, 8, 16, 256, 3, ctypes.c_void_p(0x2000), a, None, None)) == b"LCD_ERR_NULL"


def test_header_is_plain_c_and_links_from_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 and a C program must link and run
    import shutil
    import subprocess
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_lcd.c"
    src.write_text(
        '#include <stdio.h>\n#include "lcd.h"\n'
        "int main(void) {\n"
        "    if (lcd_packed_bytes(16, 256, 3) != 1536 || lcd_lut_bytes(16, 4) != 512) return 1;\n"
        "    if (lcd_pack_indices_host(NULL, 16, 256, 2, NULL, 0) != LCD_ERR_NULL) return 2;\n"
        '    printf("%s %d\\n", lcd_status_string(LCD_ERR_BAD_BITS), lcd_layout_revision());\n'
        "    return 0;\n}\n")
    exe = tmp_path / "use_lcd"
    libdir = root / "paper_2506_12038_amd"
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", f"-I{root / 'include'}", str(src), "-o", str(exe),
                           f"-L{libdir}", "-llcd", f"-Wl,-rpath,{libdir}"])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out
    assert out.stdout.split() == ["LCD_ERR_BAD_BITS", "1"]
