"""The product path has no CPU fallback: host tensors are refused by every device entry of the
binding and by the layers, and a missing library that cannot be built is an error, not a detour."""
import numpy as np
import pytest
import torch

from paper_2104_14129_amd import binding as B
from paper_2104_14129_amd import layers as L


def test_host_tensors_are_refused_before_anything_is_called():
    x = torch.zeros((2, 512))
    bits = torch.full((2,), 2, dtype=torch.uint8)
    offs = torch.zeros(2, dtype=torch.int64)
    packed = torch.zeros(256, dtype=torch.uint8)
    header = torch.zeros(2 * 2 * 2)
    calls = [
        lambda: B.group_stats(x),
        lambda: B.quantize_pack(x, bits, offs, packed, header, seed=1),
        lambda: B.unpack_dequantize(packed, header, bits, offs, x),
        lambda: B.sample_sensitivity(torch.zeros((2, 2))),
        lambda: B.allocate_bits_device(torch.ones(2), 512, 4096),
        lambda: B.tensor_stats(x),
        lambda: B.relu_forward(x, torch.empty_like(x), torch.zeros(B.relu_mask_bytes(x.numel()), dtype=torch.uint8)),
        lambda: B.maxpool2d_forward(torch.zeros((1, 4, 4)), (2, 2), (2, 2)),
        lambda: L.compress(x),
    ]
    for call in calls:
        with pytest.raises((ValueError, RuntimeError)) as err:
            call()
        assert "GPU" in str(err.value) or "cuda" in str(err.value).lower(), str(err.value)


def test_a_library_that_is_missing_and_cannot_be_built_is_an_error(monkeypatch, tmp_path):
    from paper_2104_14129_amd import build as builder

    def no_compiler(*a, **k):
        raise RuntimeError("hipcc not found: libactq cannot be built")

    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libactq.so"))
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(builder, "build", no_compiler)
    with pytest.raises(RuntimeError) as err:
        B.lib()
    assert "cannot be built" in str(err.value)
    with pytest.raises(RuntimeError):
        B.packed_bytes(1, 256, np.array([2], dtype=np.uint8))
