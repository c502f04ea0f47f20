"""GPU: the device packer/unpacker and table build against the layout definition (bit-exact)."""
import numpy as np
import pytest

import paper_2506_12038_amd as lcd
from oracle.pack_ref import pack_ref
from gpu_common import to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("shape", [(16, 256), (48, 768), (4096, 4096), (11008, 4096), (4096, 11008)])
def test_device_pack_is_bit_exact(bits, shape):
    import torch
    N, K = shape
    idx = np.random.default_rng(N + K + bits).integers(0, 1 << bits, size=(N, K), dtype=np.uint8)
    packed = lcd.lcd_pack_indices(to_dev(idx), bits)
    torch.cuda.synchronize()
    host = lcd.lcd_pack_indices_host(idx, bits)
    assert np.array_equal(packed.cpu().numpy(), host)
    if N * K <= 48 * 768:
        assert np.array_equal(host, pack_ref(idx, bits))
    else:  # sample tiles against the element-wise definition
        assert np.array_equal(lcd.lcd_pack_indices_host(idx[:32, :512], bits), pack_ref(idx[:32, :512], bits))
    back = lcd.lcd_unpack_indices(packed, N, K, bits)
    torch.cuda.synchronize()
    assert np.array_equal(back.cpu().numpy(), idx)


def test_device_pack_masks_out_of_range_indices():
    import torch
    idx = np.random.default_rng(1).integers(0, 256, size=(16, 256), dtype=np.uint8)
    for bits in (2, 3, 4):
        packed = lcd.lcd_pack_indices(to_dev(idx), bits)
        torch.cuda.synchronize()
        assert np.array_equal(packed.cpu().numpy(), lcd.lcd_pack_indices_host(idx & ((1 << bits) - 1), bits))


def test_max_size_matrix_pack_roundtrip():
    import torch
    N, K, bits = 28672, 8192, 2
    g = torch.Generator(device="cuda"); g.manual_seed(7)
    idx = torch.randint(0, 4, (N, K), dtype=torch.uint8, device="cuda", generator=g)
    packed = lcd.lcd_pack_indices(idx, bits)
    assert packed.numel() == 58720256
    back = lcd.lcd_unpack_indices(packed, N, K, bits)
    assert torch.equal(back, idx)
    # sampled tiles against the host packer
    rows = slice(16 * 1000, 16 * 1002)
    sub = idx[rows].cpu().numpy()
    hp = lcd.lcd_pack_indices_host(sub, bits)
    kc = K // 256
    got = packed[1000 * kc * 1024:(1002 * kc) * 1024].cpu().numpy()
    assert np.array_equal(got, hp)
