"""Pins for the oracle's exact layer contexts (appendix: "Activation Layers", "Pooling Layers").

ReLU keeps one bit per element, max pooling the 8-bit position of the maximum inside the
window.  Both are exact, so the pins are library routines (numpy, torch's CPU max_pool2d and
its autograd), a brute-force restatement on padded arrays, and conservation properties.
"""
import itertools

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle


# ----------------------------------------------------------------------------- ReLU

@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("n", [1, 7, 8, 255, 256, 257, 5000])
def test_relu_forward_is_numpy_where_and_little_endian_packbits(n, dtype):
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n).astype(dtype)
    x[rng.integers(0, n, n // 5 + 1)] = 0.0
    y, mask = oracle.relu_forward(x)
    assert np.array_equal(y, np.where(x > 0, x, 0).astype(dtype))
    assert mask.size == (n + 255) // 256 * 32
    bits = np.zeros(mask.size * 8, dtype=np.uint8)
    bits[:n] = x > 0
    assert np.array_equal(mask, np.packbits(bits, bitorder="little"))


def test_relu_special_values():
    x = np.array([-0.0, 0.0, np.nan, -np.inf, np.inf, 1e-45, -1e-45, 3.0], dtype=np.float32)
    y, mask = oracle.relu_forward(x)
    assert mask[0] == 0b10110000
    assert np.array_equal(y.view(np.uint32), np.array([0, 0, 0, 0, np.inf, 1e-45, 0, 3.0], dtype=np.float32).view(np.uint32))
    g = np.array([-1, np.nan, 3, -np.inf, 5, np.nan, -7, -8], dtype=np.float32)
    gx = oracle.relu_backward(mask, g)
    want = np.array([0, 0, 0, 0, 5, np.nan, 0, -8], dtype=np.float32)
    assert np.array_equal(gx.view(np.uint32), want.view(np.uint32))    # +0 where the bit is clear: a selection, not g * 0 (which would give -0 and NaN)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_relu_backward_is_the_derivative(dtype):
    rng = np.random.default_rng(3)
    n = 3000
    x = rng.standard_normal(n).astype(dtype)
    g = rng.standard_normal(n).astype(dtype)
    _, mask = oracle.relu_forward(x)
    gx = oracle.relu_backward(mask, g)
    assert np.array_equal(gx, np.where(x > 0, g, 0).astype(dtype))
    # f'(x) by central differences away from the kink
    xs = x.astype(np.float64)
    far = np.abs(xs) > 1e-2
    h = 1e-3
    fd = (np.maximum(xs + h, 0) - np.maximum(xs - h, 0)) / (2 * h)
    ones = oracle.relu_backward(mask, np.ones(n, dtype=dtype)).astype(np.float64)
    assert np.allclose(ones[far], fd[far])
    # storage: one bit per element (rounded up to whole 256-bit groups)
    assert mask.size * 8 - n < 256


# ----------------------------------------------------------------------------- max pooling

CONFIGS = [
    # H, W, kernel, stride, padding, dilation
    (112, 112, (3, 3), (2, 2), (1, 1), (1, 1)),      # the ResNet stem
    (8, 8, (2, 2), (2, 2), (0, 0), (1, 1)),
    (9, 11, (3, 2), (1, 2), (1, 0), (2, 1)),
    (7, 5, (1, 1), (1, 1), (0, 0), (1, 1)),
    (13, 17, (5, 4), (3, 2), (2, 2), (1, 2)),
    (16, 16, (16, 16), (1, 1), (0, 0), (1, 1)),      # K = 256, the largest position an 8-bit code holds
    (6, 6, (3, 3), (1, 1), (1, 1), (1, 1)),          # heavy overlap
]


def _positions_to_flat(arg, H, W, kernel, stride, padding, dilation):
    OH, OW = arg.shape[-2:]
    i = np.arange(OH)[:, None]
    j = np.arange(OW)[None, :]
    r = stride[0] * i - padding[0] + dilation[0] * (arg // kernel[1])
    c = stride[1] * j - padding[1] + dilation[1] * (arg % kernel[1])
    return r * W + c


@pytest.mark.parametrize("cfg", CONFIGS)
@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_maxpool_forward_against_torch(cfg, dtype):
    H, W, k, s, p, d = cfg
    rng = np.random.default_rng(H * 31 + W)
    x = rng.standard_normal((2, 3, H, W)).astype(dtype)
    y, arg = oracle.maxpool2d_forward(x, k, s, p, d)
    ty, tidx = F.max_pool2d(torch.from_numpy(x.astype(np.float32)), k, s, p, d, return_indices=True)
    assert y.shape == tuple(ty.shape) == x.shape[:2] + oracle.pool2d_output_size(H, W, k, s, p, d)
    assert np.array_equal(y.astype(np.float32), ty.numpy())          # max of binary16 values is exact
    assert int(arg.max()) < k[0] * k[1]
    assert np.array_equal(_positions_to_flat(arg.astype(np.int64), H, W, k, s, p, d), tidx.numpy())


@pytest.mark.parametrize("cfg", CONFIGS[:5])
def test_maxpool_forward_brute_force_on_a_padded_array(cfg):
    H, W, k, s, p, d = cfg
    rng = np.random.default_rng(5)
    x = rng.integers(-3, 4, size=(2, H, W)).astype(np.float32)        # many ties
    y, arg = oracle.maxpool2d_forward(x, k, s, p, d)
    xp = np.full((2, H + 2 * p[0], W + 2 * p[1]), -np.inf, dtype=np.float32)
    xp[:, p[0]:p[0] + H, p[1]:p[1] + W] = x
    OH, OW = y.shape[-2:]
    for n, i, j in itertools.product(range(2), range(OH), range(OW)):
        win = xp[n, s[0] * i: s[0] * i + d[0] * (k[0] - 1) + 1: d[0], s[1] * j: s[1] * j + d[1] * (k[1] - 1) + 1: d[1]]
        assert win.shape == k
        assert y[n, i, j] == win.max()
        assert arg[n, i, j] == int(np.argmax(win))                    # numpy: first maximum, row by row


def test_maxpool_ties_and_padding():
    x = np.zeros((1, 4, 4), dtype=np.float32)
    y, arg = oracle.maxpool2d_forward(x, (3, 3), (2, 2), (1, 1))
    # top-left window: rows/cols -1..1, first in-bounds position is (1,1) -> k = 4
    assert arg[0, 0, 0] == 4 and arg[0, 0, 1] == 3 and arg[0, 1, 0] == 1 and arg[0, 1, 1] == 0
    assert np.all(y == 0)
    for bad in [dict(kernel=(3, 3), stride=(2, 2), padding=(2, 2)), dict(kernel=(17, 16), stride=(1, 1)),
                dict(kernel=(2, 2), stride=(0, 1)), dict(kernel=(5, 5), stride=(1, 1))]:
        with pytest.raises(oracle.OracleError):
            oracle.maxpool2d_forward(x, **bad)


@pytest.mark.parametrize("cfg", CONFIGS)
def test_maxpool_backward_against_torch_autograd(cfg):
    H, W, k, s, p, d = cfg
    rng = np.random.default_rng(H + 7 * W)
    x = rng.standard_normal((2, 2, H, W)).astype(np.float32)
    y, arg = oracle.maxpool2d_forward(x, k, s, p, d)
    for integer in (True, False):
        gy = (rng.integers(-8, 9, size=y.shape) if integer else rng.standard_normal(y.shape)).astype(np.float32)
        gx = oracle.maxpool2d_backward(arg, gy, H, W, k, s, p, d)
        tx = torch.from_numpy(x).requires_grad_(True)
        F.max_pool2d(tx, k, s, p, d).backward(torch.from_numpy(gy))
        if integer:                                                    # small integers: every sum is exact
            assert np.array_equal(gx, tx.grad.numpy())
            assert gx.sum() == gy.sum()
        else:
            assert np.allclose(gx, tx.grad.numpy(), rtol=1e-6, atol=1e-6)
    # binary16 gradients: accumulated in binary32, rounded once
    gy16 = rng.standard_normal(y.shape).astype(np.float16)
    gx16 = oracle.maxpool2d_backward(arg, gy16, H, W, k, s, p, d)
    ref = oracle.maxpool2d_backward(arg, gy16.astype(np.float32), H, W, k, s, p, d)
    assert np.array_equal(gx16, ref.astype(np.float16))


def test_maxpool_backward_rejects_positions_the_forward_cannot_produce():
    x = np.random.default_rng(0).standard_normal((1, 6, 6)).astype(np.float32)
    y, arg = oracle.maxpool2d_forward(x, (3, 3), (2, 2), (1, 1))
    gy = np.ones_like(y)
    bad = arg.copy()
    bad[0, 0, 0] = 0                       # points at the padding
    with pytest.raises(oracle.OracleError):
        oracle.maxpool2d_backward(bad, gy, 6, 6, (3, 3), (2, 2), (1, 1))
    bad = arg.copy()
    bad[0, 1, 1] = 9                       # outside the window
    with pytest.raises(oracle.OracleError):
        oracle.maxpool2d_backward(bad, gy, 6, 6, (3, 3), (2, 2), (1, 1))


def test_context_sizes_of_the_resnet_stem():
    """ReLU: 1 bit per element; max pooling: 8 bits per OUTPUT location, i.e. 2 bits per input
    element at stride 2 -- both small beside the 32-bit activations they replace."""
    N, C, H, W = 2, 4, 112, 112
    x = np.random.default_rng(1).standard_normal((N, C, H, W)).astype(np.float32)
    _, mask = oracle.relu_forward(x)
    assert mask.size * 8 == x.size
    y, arg = oracle.maxpool2d_forward(x, (3, 3), (2, 2), (1, 1))
    assert arg.dtype == np.uint8 and arg.size * 4 == x.size
