"""The binding refuses buffers that are too short or of the wrong element type before the
library is called: a kernel writing past an allocation is a GPU fault, not an exception.
Host-only: the checks run before any device work, on CPU tensors standing in for the
arguments (which the binding rejects for not being on the device only after the size and
type checks would have passed)."""
import pytest
import torch

from paper_2306_10209_amd import binding as zpp


class FakeDev(torch.Tensor):
    """A CPU tensor that claims to be on the device: enough for the checks that run before
    the library is called (nothing here reaches a launch: every case must raise first)."""
    @property
    def is_cuda(self):
        return True


def fake(n, dtype):
    return torch.empty(n, dtype=dtype).as_subclass(FakeDev)


def test_short_or_mistyped_outputs_raise():
    x = fake(4096, torch.float16)
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qwz_quantize(x, 256, 8, codes=fake(4095, torch.uint8), scales=fake(16, torch.float32))
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qwz_quantize(x, 256, 8, codes=fake(4096, torch.uint8), scales=fake(15, torch.float32))
    with pytest.raises(zpp.ZppError, match="dtype"):
        zpp.qwz_quantize(x, 256, 8, codes=fake(4096, torch.uint8), scales=fake(16, torch.float16))
    with pytest.raises(zpp.ZppError, match="dtype"):
        zpp.qwz_quantize(x, 256, 8, codes=fake(4096, torch.int32), scales=fake(16, torch.float32))
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qwz_dequantize(fake(4096, torch.uint8), fake(16, torch.float32), 4096, 256, 8, out=fake(4000, torch.float16))
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qwz_dequantize(fake(2047, torch.uint8), fake(16, torch.float32), 4096, 256, 4, out=fake(4096, torch.float16))
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qgz_reorder(x, 2, 2, 1, 256, 4, codes=fake(2047, torch.uint8), scales=fake(16, torch.float32))


def test_short_peer_buffers_and_outputs_raise():
    m, B = 2048, 512
    good = [fake(m // 2, torch.uint8) for _ in range(3)], [fake(m // B, torch.float32) for _ in range(3)]
    short_codes = [fake(m // 2, torch.uint8), fake(m // 2 - 1, torch.uint8)], [fake(m // B, torch.float32)] * 2
    short_scales = [fake(m // 2, torch.uint8)] * 2, [fake(m // B, torch.float32), fake(m // B - 1, torch.float32)]
    for bad in (short_codes, short_scales):
        with pytest.raises(zpp.ZppError, match="shorter"):
            zpp.qgz_intra_reduce(bad[0], bad[1], m, B, 4, codes_out=fake(m // 2, torch.uint8), scales_out=fake(m // B, torch.float32))
        with pytest.raises(zpp.ZppError, match="shorter"):
            zpp.qgz_inter_reduce(bad[0], bad[1], m, B, 4, 2.0, out=fake(m, torch.float32))
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qgz_intra_reduce(good[0], good[1], m, B, 4, codes_out=fake(m // 2 - 16, torch.uint8), scales_out=fake(m // B, torch.float32))
    with pytest.raises(zpp.ZppError, match="needs"):
        zpp.qgz_inter_reduce(good[0], good[1], m, B, 4, 2.0, out=fake(m - 1, torch.float32))
    with pytest.raises(zpp.ZppError, match="dtype"):
        zpp.qgz_inter_reduce(good[0], good[1], m, B, 4, 2.0, out=fake(m, torch.float16))
    with pytest.raises(zpp.ZppError, match="dtype"):
        zpp.PeerTable([fake(8, torch.uint8)], [fake(8, torch.float16)])
    with pytest.raises(zpp.ZppError, match="length"):
        zpp.PeerTable(good[0], good[1][:2])
