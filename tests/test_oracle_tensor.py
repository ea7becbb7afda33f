"""Pins for the oracle's per-tensor quantizer (one range and zero point for the whole tensor:
the baseline of Sec. 4.1's variance argument and of Sec. 6.1's ablation), and the argument
itself: on heterogeneous group ranges the per-group quantizer has a far smaller variance."""
import numpy as np
import pytest

import oracle


def test_tensor_stats_is_numpy_min_and_max_minus_min():
    rng = np.random.default_rng(0)
    for dtype in (np.float32, np.float16):
        x = (rng.standard_normal((5, 1000)) * 7 - 2).astype(dtype)
        zr = oracle.tensor_stats(x)
        x32 = x.astype(np.float32)
        assert zr[0] == x32.min() and zr[1] == np.float32(x32.max() - x32.min())
    z = oracle.tensor_stats(np.array([[0.0, -0.0, 3.0]], dtype=np.float32))
    assert z[0] == 0 and not np.signbit(z[0])


@pytest.mark.parametrize("noise_bits", [24, 16])
@pytest.mark.parametrize("b", [1, 2, 3, 4, 8])
def test_equals_the_per_group_quantizer_when_every_group_spans_the_tensor_range(b, noise_bits):
    """If each group contains the global minimum and maximum, per-group (Z, R) equal the
    per-tensor ones, so codes and dequantized values must coincide with the pinned
    per-group path."""
    rng = np.random.default_rng(b)
    N, D = 3, 256 * 4
    x = rng.uniform(-1, 2, (N, D)).astype(np.float32)
    x.reshape(N, 4, 256)[:, :, 7] = -1.5
    x.reshape(N, 4, 256)[:, :, 99] = 2.25
    bits = np.full(N, b, dtype=np.uint8)
    zr = oracle.tensor_stats(x)
    assert zr[0] == np.float32(-1.5) and zr[1] == np.float32(3.75)
    packed_t, off_t = oracle.quantize_pack_tensor(x, bits, zr, seed=4, tag=9, noise_bits=noise_bits)
    packed_g, header_g, off_g = oracle.quantize_pack(x, bits, 4, 9, noise_bits=noise_bits)
    assert np.array_equal(off_t, off_g) and np.array_equal(packed_t, packed_g)
    out_t = oracle.unpack_dequantize_tensor(packed_t, zr, bits, off_t, N, D)
    out_g = oracle.unpack_dequantize(packed_g, header_g, bits, off_g, N, D)
    assert np.array_equal(out_t.view(np.uint32), out_g.view(np.uint32))


def test_mixed_widths_ragged_tail_and_binary16():
    rng = np.random.default_rng(5)
    N, D = 4, 256 * 3 + 77
    x = rng.standard_normal((N, D)).astype(np.float16)
    bits = np.array([1, 3, 4, 8], dtype=np.uint8)
    zr = oracle.tensor_stats(x)
    packed, off = oracle.quantize_pack_tensor(x, bits, zr, seed=1, noise_bits=16)
    out = oracle.unpack_dequantize_tensor(packed, zr, bits, off, N, D, out_dtype=np.float16)
    # every value lands on the tensor-wide grid of its sample's width, within one step of the input
    for n in range(N):
        B = (1 << int(bits[n])) - 1
        step = float(zr[1]) / B
        err = np.abs(out[n].astype(np.float64) - x[n].astype(np.float64))
        assert err.max() <= step * (1 + 1e-3) + 1e-3
    # padding codes of the ragged last group are zero
    ng = 4
    last = packed[int(off[3]) + 3 * 256: int(off[3]) + 4 * 256]
    assert np.all(last[77:] == 0)


def test_constant_tensor_is_degenerate():
    x = np.full((2, 512), 1.25, dtype=np.float32)
    zr = oracle.tensor_stats(x)
    assert zr[1] == 0
    bits = np.full(2, 2, dtype=np.uint8)
    packed, off = oracle.quantize_pack_tensor(x, bits, zr, seed=3)
    assert not packed.any()
    assert np.all(oracle.unpack_dequantize_tensor(packed, zr, bits, off, 2, 512) == 1.25)


def _expected_variance(x, z, scale, B):
    """Exact variance of stochastic rounding per element: scale^2 * p (1 - p), p = frac(u)."""
    u = (x.astype(np.float64) - z) / np.where(scale > 0, scale, 1.0)
    p = u - np.floor(u)
    return (scale.astype(np.float64) ** 2) * p * (1 - p)


@pytest.mark.parametrize("b", [2, 4])
def test_unbiased_with_the_closed_form_variance(b):
    rng = np.random.default_rng(11)
    N, D = 2, 512
    x = rng.standard_normal((N, D)).astype(np.float32)
    bits = np.full(N, b, dtype=np.uint8)
    zr = oracle.tensor_stats(x)
    B = (1 << b) - 1
    S = 1500
    acc = np.zeros((N, D)); acc2 = np.zeros((N, D))
    for s in range(S):
        packed, off = oracle.quantize_pack_tensor(x, bits, zr, seed=1000 + s, noise_bits=16)
        out = oracle.unpack_dequantize_tensor(packed, zr, bits, off, N, D).astype(np.float64)
        acc += out; acc2 += out * out
    mean = acc / S
    var = acc2 / S - mean ** 2
    scale = np.float32(zr[1]) / np.float32(B)
    want = _expected_variance(x, zr[0], np.full((N, D), scale, dtype=np.float32), B)
    z = (mean - x) / np.sqrt(np.maximum(want, 1e-30) / S)
    assert np.abs(z[want > 1e-12]).max() < 5.5
    assert abs(var.sum() / want.sum() - 1) < 0.03


def test_per_group_variance_is_far_below_per_tensor_on_heterogeneous_ranges():
    """The argument of Sec. 4.1: with one range for the tensor every group pays for the largest
    range, R^2 G / (6 B^2), while per-group ranges pay only for their own.  Group ranges spread
    over orders of magnitude (the heterogeneity the paper reports); expected variances from the
    closed form, one Monte-Carlo spot check."""
    rng = np.random.default_rng(21)
    N, ng, G = 8, 32, 256
    sigma = np.exp(rng.normal(0, 1.5, (N, ng, 1)))                  # heterogeneous group scales
    x = (rng.standard_normal((N, ng, G)) * sigma).astype(np.float32).reshape(N, ng * G)
    gmin, grange = oracle.group_stats(x)
    zr = oracle.tensor_stats(x)
    ratios = {}
    for b in (1, 2, 3, 4, 8):
        B = (1 << b) - 1
        pg_scale = np.repeat((grange / np.float32(B)), G, axis=1)
        pg_z = np.repeat(gmin, G, axis=1)
        v_pg = _expected_variance(x, pg_z, pg_scale, B).sum()
        v_pt = _expected_variance(x, zr[0], np.full(x.shape, np.float32(zr[1]) / np.float32(B), dtype=np.float32), B).sum()
        ratios[b] = v_pt / v_pg
        # the rule of thumb R^2 G / (6 B^2) summed over groups, within a factor of two
        approx_pg = (grange.astype(np.float64) ** 2).sum() * G / (6 * B * B)
        if b >= 3:
            assert 0.5 < v_pg / approx_pg < 2.0
    assert all(r > 10 for r in ratios.values()), ratios
    # per-group at b bits beats per-tensor at b + 2 bits here
    # spot check of the expectation by sampling, b = 2
    bits = np.full(N, 2, dtype=np.uint8)
    S = 200
    se_pt = se_pg = 0.0
    for s in range(S):
        pk, off = oracle.quantize_pack_tensor(x, bits, zr, seed=s, noise_bits=16)
        se_pt += ((oracle.unpack_dequantize_tensor(pk, zr, bits, off, N, ng * G).astype(np.float64) - x) ** 2).sum()
        pk, hd, off = oracle.quantize_pack(x, bits, s, 0, noise_bits=16)
        se_pg += ((oracle.unpack_dequantize(pk, hd, bits, off, N, ng * G).astype(np.float64) - x) ** 2).sum()
    assert abs((se_pt / se_pg) / ratios[2] - 1) < 0.1
