"""GPU: the allocation-free decode entry point (lcd_lut_gemv_noalloc) against lcd_lut_gemv.

Two calls in a row on one GPU share the library's static scratch array, the second with a smaller
input than the first; each must reproduce lcd_lut_gemv bit for bit (both routes round the same way)
and match the oracle.  The device-memory counters of the allocator and of the driver are read around
the calls: neither may move.
"""
import numpy as np
import pytest

import oracle
import synth
import paper_2506_12038_amd as lcd
from gpu_common import TOL, assert_parity, to_dev

pytestmark = pytest.mark.gpu


def _prepare(N, K, bits, M, seed_offset):
    import torch
    layer = synth.make_layer(2, 0, N, K, bits, M, seed_offset=seed_offset)
    packed = lcd.lcd_pack_indices(to_dev(layer["idx"]), bits)
    lut = lcd.lcd_build_lut(to_dev(layer["codebook"]), bits)
    x, s = to_dev(layer["x"]), to_dev(layer["s"])
    ref = lcd.lcd_lut_gemv(packed, lut, x, s, N, bits)
    y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
    Y = oracle.lut_matmul(layer["codebook"], layer["idx"], layer["x"], layer["s"], bits)
    return dict(packed=packed, lut=lut, x=x, s=s, ref=ref, y=y, Y=Y, N=N, bits=bits)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_two_calls_in_a_row_the_second_smaller(bits):
    import torch
    # the first call fills the whole scratch array (16 tokens x 32768 columns), the second uses a corner of it
    big = _prepare(48, 32768, bits, 16, 1)
    small = _prepare(80, 1280, bits, 3, 2)
    one = _prepare(64, 2304, bits, 1, 3)
    torch.cuda.synchronize()
    lcd.lcd_lut_gemv_noalloc(big["packed"], big["lut"], big["x"], big["s"], big["N"], bits, big["y"])   # first call on the device: address look-up
    torch.cuda.synchronize()
    big["y"].fill_(float("nan"))
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    reserved0 = torch.cuda.memory_reserved()
    for c in (big, small, one):
        lcd.lcd_lut_gemv_noalloc(c["packed"], c["lut"], c["x"], c["s"], c["N"], bits, c["y"])
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0 and torch.cuda.memory_reserved() == reserved0
    for c in (big, small, one):
        assert torch.equal(c["y"], c["ref"])
        assert_parity(c["y"].cpu().numpy(), c["Y"], TOL)


def test_sizes_beyond_the_static_scratch_are_rejected():
    import torch
    bits, N = 2, 16
    for M, K, ok in ((16, 32768, True), (16, 33024, False), (8, 65536, True), (9, 65536, False), (1, 262144, True)):
        packed = torch.zeros(lcd.lcd_packed_bytes(N, K, bits), dtype=torch.uint8, device="cuda")
        lut = lcd.lcd_build_lut(torch.zeros((N, 4), dtype=torch.float16, device="cuda"), bits)
        x = torch.zeros((M, K), dtype=torch.float16, device="cuda")
        s = torch.ones(K, dtype=torch.float32, device="cuda")
        y = torch.full((M, N), float("nan"), dtype=torch.float16, device="cuda")
        if ok:
            lcd.lcd_lut_gemv_noalloc(packed, lut, x, s, N, bits, y)
            torch.cuda.synchronize()
            assert torch.equal(y, torch.zeros_like(y))
        else:
            with pytest.raises(lcd.LcdError) as e:
                lcd.lcd_lut_gemv_noalloc(packed, lut, x, s, N, bits, y)
            assert e.value.name == "LCD_ERR_SIZE" and "static scratch" in str(e.value)
            torch.cuda.synchronize()
            assert bool(torch.isnan(y).all())      # nothing was launched
    with pytest.raises(lcd.LcdError) as e:
        lcd.lcd_lut_gemv_noalloc(packed, lut, torch.zeros((17, 256), dtype=torch.float16, device="cuda"),
                                 torch.ones(256, dtype=torch.float32, device="cuda"), N, bits,
                                 torch.zeros((17, N), dtype=torch.float16, device="cuda"))
    assert e.value.name == "LCD_ERR_BAD_M"


def test_replayed_from_a_hip_graph():
    # the callers this entry point is for: captured once (after a first call outside capture), replayed
    # with eager work in between; every replay reproduces the eager result
    import torch
    bits = 3
    c = _prepare(96, 4352, bits, 5, 4)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        lcd.lcd_lut_gemv_noalloc(c["packed"], c["lut"], c["x"], c["s"], c["N"], bits, c["y"], stream=stream)
    torch.cuda.synchronize()
    assert torch.equal(c["y"], c["ref"])
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        lcd.lcd_lut_gemv_noalloc(c["packed"], c["lut"], c["x"], c["s"], c["N"], bits, c["y"], stream=stream)
    for rep in range(3):
        c["y"].fill_(float("nan"))
        torch.cuda.synchronize()
        with torch.cuda.stream(stream):
            graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(c["y"], c["ref"]), rep
