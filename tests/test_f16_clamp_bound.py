"""The binary16 quantizer with 16-bit noise leaves out the clamp of the scaled value for widths
below 8 bits.  That is sound if, for every range r a binary16 group can have, the largest scaled
value fl32(r * fl32(B / r)) plus the largest noise (1 - 2^-16), rounded to binary32, stays below
B + 1 (Sec. 4.1 scaling; every other element of the group scales to no more than the maximum does,
by monotonicity of rounding).  Checked here on every range with Z = 0 (all positive binary16
numbers) and on a million random (Z, maximum) pairs; for 8 bits the same computation must find
ranges that do reach 256, or the kernel's remaining clamp would be dead code."""
import numpy as np
import pytest


def _worst_sum(r32: np.ndarray, b: int) -> np.ndarray:
    B = np.float32((1 << b) - 1)
    q = (B / r32).astype(np.float32)
    s = (r32 * q).astype(np.float32)
    # one rounding of the exact sum, as a fused multiply-add does (the sum is exact in binary64)
    return (s.astype(np.float64) + (65535.0 / 65536.0)).astype(np.float32)


def _ranges() -> np.ndarray:
    pos = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float32)
    rng = np.random.default_rng(5)
    a = rng.integers(0, 0x7C00, 1_000_000).astype(np.uint16)
    c = rng.integers(0, 0x7C00, 1_000_000).astype(np.uint16)
    sa = np.where(rng.integers(0, 2, a.size) == 1, np.uint16(0x8000), np.uint16(0))
    sc = np.where(rng.integers(0, 2, a.size) == 1, np.uint16(0x8000), np.uint16(0))
    fa = (a | sa).view(np.float16).astype(np.float32)
    fc = (c | sc).view(np.float16).astype(np.float32)
    diff = (np.maximum(fa, fc) - np.minimum(fa, fc)).astype(np.float32)
    return np.concatenate([pos, diff[diff > 0]])


@pytest.mark.parametrize("b", [1, 2, 3, 4, 5, 6, 7])
def test_no_range_reaches_the_next_code_below_8_bits(b):
    assert np.all(_worst_sum(_ranges(), b) < np.float32(1 << b))


def test_at_8_bits_some_ranges_do():
    assert np.any(_worst_sum(_ranges(), 8) >= np.float32(256.0))
