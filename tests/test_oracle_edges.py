"""Further pins of the oracle, each aimed at a mistake that the other pin files would let through
(found by changing the oracle's source one operator or constant at a time and running the pins):
sizes that leave one element in the last group, noise indices beyond the first group in the
bfloat16-header mode, the strictness of the rounding comparison, stream bytes that no code
touches, invalid widths and positions, and the edge cases of the binary16 conversion."""
import numpy as np
import pytest

import oracle

G = 256


def _bf(h):
    return (np.asarray(h, dtype=np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------- D = k G + 1

def test_one_element_in_the_last_group():
    """ng = ceil(D / G): with D = 2 G + 1 there are three groups, the last one a single element
    (range 0, code 0, reconstructed exactly)."""
    rng = np.random.default_rng(0)
    N, D = 3, 2 * G + 1
    x = rng.standard_normal((N, D)).astype(np.float32)
    x[:, -1] = [0.5, -2.0, 3.140625]       # bfloat16 values, so that the lone element is exact in both header formats
    bits = np.array([2, 3, 8], dtype=np.uint8)
    offsets, total = oracle.packed_bytes(N, D, G, bits)
    assert total == 3 * 32 * (2 + 3 + 8) and list(offsets) == [0, 3 * 32 * 2, 3 * 32 * 5]   # Sec. 5.1 stream: ng * G * b / 8
    gmin, grange = oracle.group_stats(x)
    assert gmin.shape == (N, 3)
    assert np.array_equal(gmin[:, 2], x[:, -1]) and np.all(grange[:, 2] == 0)
    assert np.array_equal(gmin[:, :2], x[:, :2 * G].reshape(N, 2, G).min(axis=2))
    packed, header, off = oracle.quantize_pack(x, bits, seed=5, noise_bits=16)
    assert header.shape == (N, 3, 2)
    assert np.array_equal(header[:, 2, 0], x[:, -1]) and np.all(header[:, 2, 1] == 0)
    out = oracle.unpack_dequantize(packed, header, bits, off, N, D)
    assert np.array_equal(out[:, -1], x[:, -1])
    for n in range(N):     # the single element's code and the 255 padding codes are zero
        last = packed[int(off[n]) + 2 * 32 * int(bits[n]): int(off[n]) + 3 * 32 * int(bits[n])]
        assert not last.any()
    codes = oracle.quantize_codes(x, bits, seed=5, noise_bits=16)
    assert codes.shape == (N, D) and np.all(codes[:, -1] == 0)
    # bfloat16 header: the lone element's group stores Z = its value and R = 0
    p16, h16, off16 = oracle.quantize_pack_bf16(x, bits, seed=5, noise_bits=16)
    assert h16.shape == (N, 3, 2) and np.all(h16[:, 2, 1] == 0)
    assert np.array_equal(_bf(h16[:, 2, 0]), x[:, -1])
    o16 = oracle.unpack_dequantize_bf16(p16, h16, bits, off16, N, D)
    assert o16.shape == (N, D) and np.array_equal(o16[:, -1], x[:, -1])
    # sensitivities sum over all three groups
    w = oracle.sample_sensitivity(np.abs(rng.standard_normal((N, 3))).astype(np.float32))
    assert w.shape == (N,)


# ----------------------------------------------------------------------------- bfloat16-header mode

@pytest.mark.parametrize("noise_bits", [16, 24])
def test_bf16_mode_equals_fp32_mode_when_the_headers_are_exact(noise_bits):
    """Minimum and range of every group are bfloat16 values, so rounding the header changes
    nothing: codes and reconstructions of the two modes must coincide bit for bit -- over several
    samples, several groups, mixed widths and a ragged tail, with values off the grid so that
    every code depends on its own noise word."""
    rng = np.random.default_rng(11)
    N, D = 3, 3 * G + 100
    x = rng.uniform(-1.5, 2.5, (N, D)).astype(np.float32)
    for g in range(4):                      # -1.5 and 2.5 in every group: Z = -1.5, R = 4
        lo = g * G
        x[:, lo + 3] = -1.5
        x[:, lo + 41] = 2.5
    bits = np.array([2, 5, 8], dtype=np.uint8)
    p16, h16, off16 = oracle.quantize_pack_bf16(x, bits, seed=9, tag=2, noise_bits=noise_bits)
    p32, h32, off32 = oracle.quantize_pack(x, bits, seed=9, tag=2, noise_bits=noise_bits)
    assert np.all(_bf(h16[:, :, 0]) == -1.5) and np.all(_bf(h16[:, :, 1]) == 4.0)
    assert np.array_equal(off16, off32)
    assert np.array_equal(p16, p32)
    codes = oracle.quantize_codes(x, bits, seed=9, tag=2, noise_bits=noise_bits)
    assert len(np.unique(codes[2])) > 100   # the comparison is not vacuous: the codes vary
    o16 = oracle.unpack_dequantize_bf16(p16, h16, bits, off16, N, D)
    o32 = oracle.unpack_dequantize(p32, h32, bits, off32, N, D)
    assert np.array_equal(o16.view(np.uint32), o32.view(np.uint32))
    # and the noise really is indexed by (sample, feature): moving a sample moves its codes
    p_swapped, _, _ = oracle.quantize_pack_bf16(x[::-1].copy(), bits[::-1].copy(), seed=9, tag=2, noise_bits=noise_bits)
    n_bytes = 4 * 32 * int(bits[2])
    assert not np.array_equal(p_swapped[:n_bytes], p16[int(off16[2]): int(off16[2]) + n_bytes])


# ----------------------------------------------------------------------------- per-tensor mode

@pytest.mark.parametrize("noise_bits", [16, 24])
def test_per_tensor_mode_with_one_element_in_the_last_group(noise_bits):
    """As the full-group comparison with the per-group path, with D = 3 G + 1: the single last
    element is the global minimum, which both paths encode as 0 and reconstruct exactly."""
    rng = np.random.default_rng(3)
    N, D = 2, 3 * G + 1
    x = rng.uniform(-1, 2, (N, D)).astype(np.float32)
    for g in range(3):
        x[:, g * G + 7] = -1.5
        x[:, g * G + 99] = 2.25
    x[:, -1] = -1.5
    bits = np.array([3, 8], dtype=np.uint8)
    zr = oracle.tensor_stats(x)
    packed_t, off_t = oracle.quantize_pack_tensor(x, bits, zr, seed=4, tag=9, noise_bits=noise_bits)
    packed_g, header_g, off_g = oracle.quantize_pack(x, bits, 4, 9, noise_bits=noise_bits)
    assert np.array_equal(off_t, off_g) and np.array_equal(packed_t, packed_g)
    out_t = oracle.unpack_dequantize_tensor(packed_t, zr, bits, off_t, N, D)
    out_g = oracle.unpack_dequantize(packed_g, header_g, bits, off_g, N, D)
    assert out_t.shape == (N, D)
    assert np.array_equal(out_t.view(np.uint32), out_g.view(np.uint32))


# ----------------------------------------------------------------------------- rounding rule

def test_rounding_up_needs_noise_strictly_below_the_fraction():
    """Sec. 4.1: round up with probability frac(u).  On a grid of 2^24 noise values k / 2^24 that
    is `noise < frac`: exactly frac * 2^24 of them.  An element whose fraction equals its own
    noise word therefore rounds down; one ulp more and it rounds up."""
    seed, tag, b = 21, 0, 1
    x = np.zeros((1, G), dtype=np.float32)
    x[0, 1] = 1.0                                 # Z = 0, R = 1, B = 1: u = x
    picked = 0
    for d in range(2, G):
        noise = oracle.noise(seed, tag, 0, d, 24)
        if 0.01 < noise < 0.99:
            x[0, d] = np.float32(noise) if d % 2 == 0 else np.nextafter(np.float32(noise), np.float32(1))
            picked += 1
    assert picked > 200
    codes = oracle.quantize_codes(x, np.array([b], dtype=np.uint8), seed, tag, noise_bits=24)[0]
    for d in range(2, G):
        if x[0, d] != 0:
            assert codes[d] == (0 if d % 2 == 0 else 1), d


# ----------------------------------------------------------------------------- invalid input

@pytest.mark.parametrize("b", [0, 9, 255])
def test_widths_outside_1_to_8_are_refused(b):
    x = np.zeros((2, G), dtype=np.float32)
    bits = np.array([2, b], dtype=np.uint8)
    for call in (lambda: oracle.quantize_pack(x, bits, seed=1),
                 lambda: oracle.quantize_pack_bf16(x, bits, seed=1),
                 lambda: oracle.quantize_codes(x, bits, seed=1)):
        with pytest.raises(oracle.OracleError) as err:
            call()
        assert err.value.code == oracle.EINVAL


def test_pooling_positions_outside_the_input_are_refused_one_condition_at_a_time():
    """3x3 window, stride 2, padding 1 on a 4x4 plane (2x2 outputs).  A stored position is valid
    only if it lies inside the input; each border is probed alone."""
    H = W = 4
    k, s, p = (3, 3), (2, 2), (1, 1)
    g = np.ones((1, 2, 2), dtype=np.float32)
    ok = np.full((1, 2, 2), 4, dtype=np.uint8)              # the window's centre: always inside
    assert oracle.maxpool2d_backward(ok, g, H, W, k, s, p).sum() == 4

    def refused(i, j, code):
        a = ok.copy()
        a[0, i, j] = code
        with pytest.raises(oracle.OracleError) as err:
            oracle.maxpool2d_backward(a, g, H, W, k, s, p)
        return err.value.code == oracle.EINVAL

    assert refused(0, 1, 1)      # output (0, 1), window row 0: input row -1, column 2
    assert refused(1, 0, 3)      # output (1, 0), window column 0: input row 2, column -1
    assert refused(0, 0, 9)      # beyond the 9 positions of the window
    # on a 3x3 plane the last window reaches one past the last row / column
    H = W = 3
    ok3 = np.full((1, 2, 2), 4, dtype=np.uint8)
    assert oracle.maxpool2d_backward(ok3, g, H, W, k, s, p).sum() == 4
    for (i, j, code) in ((1, 0, 7), (0, 1, 5)):    # row 3 = H with a valid column; column 3 = W with a valid row
        a = ok3.copy()
        a[0, i, j] = code
        with pytest.raises(oracle.OracleError):
            oracle.maxpool2d_backward(a, g, H, W, k, s, p)
    # the last row and column themselves are accepted
    a = ok3.copy()
    a[0, 1, 1] = 4               # output (1, 1), window centre: input (2, 2) = (H - 1, W - 1)
    a[0, 0, 1] = 3               # output (0, 1), window (1, 0): input (0, 1)
    gx = oracle.maxpool2d_backward(a, g, H, W, k, s, p)
    assert gx[0, 2, 2] == 1 and gx[0, 0, 1] == 1


_GOOD = dict(H=8, W=8, kh=3, kw=3, sh=2, sw=2, ph=1, pw=1, dh=1, dw=1)


def _pool(**change):
    a = dict(_GOOD, **change)
    return oracle.pool2d_output_size(a["H"], a["W"], (a["kh"], a["kw"]), (a["sh"], a["sw"]), (a["ph"], a["pw"]),
                                     (a["dh"], a["dw"]))


@pytest.mark.parametrize("change", [dict(H=0), dict(W=0), dict(kh=0), dict(kw=0), dict(sh=0), dict(sw=0),
                                    dict(dh=0), dict(dw=0), dict(ph=-1), dict(pw=-1), dict(ph=2), dict(pw=2),
                                    dict(kh=17, kw=16, H=40, W=40), dict(H=1, W=1, ph=0, pw=0)])
def test_pooling_geometry_is_validated_one_condition_at_a_time(change):
    """Extents, window, stride and dilation are positive, padding is non-negative and at most half
    the window, the window has at most 256 positions (they are stored in a byte), and there is
    at least one output."""
    assert _pool() == (4, 4)
    with pytest.raises(oracle.OracleError) as err:
        _pool(**change)
    assert err.value.code == oracle.EINVAL


def test_pooling_geometry_limits_that_are_allowed():
    assert _pool(kh=2, kw=2, ph=1, pw=1) == (5, 5)                    # padding of exactly half the window
    assert _pool(kh=16, kw=16, ph=0, pw=0, H=16, W=17, sh=1, sw=1) == (1, 2)   # 256 positions
    assert _pool(H=1, W=1) == (1, 1)                                  # one input element, window mostly padding


# ----------------------------------------------------------------------------- binary16 conversion

def test_float_to_half_special_values():
    assert oracle.float_to_half(65504.0) == 0x7BFF                   # the largest finite value
    assert oracle.float_to_half(65519.996) == 0x7BFF                 # below the midpoint to 65536
    assert oracle.float_to_half(65520.0) == 0x7C00                   # the midpoint ties to even: infinity
    assert oracle.float_to_half(-65520.0) == 0xFC00
    assert oracle.float_to_half(float("inf")) == 0x7C00
    h = oracle.float_to_half(float("nan"))
    assert (h & 0x7C00) == 0x7C00 and (h & 0x03FF) != 0              # a NaN stays a NaN
    assert oracle.float_to_half(2.0 ** -14) == 0x0400                # the smallest normal
    assert oracle.float_to_half(2.0 ** -24) == 0x0001                # the smallest subnormal
    assert oracle.float_to_half(2.0 ** -25) == 0x0000                # its half ties to even: zero
    assert oracle.float_to_half(1.5 * 2.0 ** -24) == 0x0002          # ties to even upwards
    want = np.array([1e-3, 0.1, 1.0 / 3.0, 1000.7, 6.1e-5, 5.9e-8], dtype=np.float32)
    got = np.array([oracle.float_to_half(float(v)) for v in want], dtype=np.uint16)
    assert np.array_equal(got, want.astype(np.float16).view(np.uint16))
