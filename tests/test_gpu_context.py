"""Parity of the exact layer contexts (ReLU bit mask, max-pooling positions) with the oracle,
through the C ABI.  Everything is compared bit for bit: masks, positions, outputs, gradients."""
import numpy as np
import pytest
import torch

import oracle
from paper_2104_14129_amd import binding as B

pytestmark = pytest.mark.gpu

CANARY = 0xA5
NP = {np.float32: torch.float32, np.float16: torch.float16}


def _bits_equal(a, b):
    return np.array_equal(np.ascontiguousarray(a).view(np.uint8), np.ascontiguousarray(b).view(np.uint8))


def _relu_round_trip(x_np, g_np, in_place=False):
    n = x_np.size
    dev = torch.device("cuda:0")
    pad = 64
    xbuf = torch.full((n + pad,), 7.0, dtype=NP[x_np.dtype.type], device=dev)
    xbuf[:n] = torch.from_numpy(x_np.reshape(-1)).to(dev)
    x = xbuf[:n]
    mbytes = B.relu_mask_bytes(n)
    mbuf = torch.full((mbytes + 256,), CANARY, dtype=torch.uint8, device=dev)
    ybuf = xbuf if in_place else torch.full((n + pad,), float("nan"), dtype=x.dtype, device=dev)
    B.relu_forward(x, ybuf[:n], mbuf[:mbytes])
    torch.cuda.synchronize()
    oy, omask = oracle.relu_forward(x_np.reshape(-1))
    assert (mbuf[mbytes:] == CANARY).all(), "relu_forward wrote past the mask"
    if in_place:
        assert (xbuf[n:] == 7.0).all()
    else:
        assert torch.isnan(ybuf[n:]).all(), "relu_forward wrote past y"
    assert np.array_equal(mbuf[:mbytes].cpu().numpy(), omask)
    assert _bits_equal(ybuf[:n].cpu().numpy(), oy)
    gbuf = torch.full((n + pad,), float("nan"), dtype=x.dtype, device=dev)
    gy = torch.from_numpy(g_np.reshape(-1)).to(dev)
    if in_place:
        gbuf[:n] = gy
        B.relu_backward(mbuf[:mbytes], gbuf[:n], gbuf[:n])
    else:
        B.relu_backward(mbuf[:mbytes], gy, gbuf[:n])
    torch.cuda.synchronize()
    assert torch.isnan(gbuf[n:]).all(), "relu_backward wrote past grad_x"
    assert _bits_equal(gbuf[:n].cpu().numpy(), oracle.relu_backward(omask, g_np.reshape(-1)))


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("n", [1, 3, 255, 256, 257, 1023, 1024, 1025, 2047, 2048, 2049, 4096 * 5, 4096 * 37 + 1999])
def test_relu_sizes_spanning_tiles_and_ragged_tails(n, dtype):
    rng = np.random.default_rng(n)
    x = rng.standard_normal(n).astype(dtype)
    x[rng.integers(0, n, n // 7 + 1)] = 0.0
    x[rng.integers(0, n, n // 9 + 1)] = -0.0
    g = rng.standard_normal(n).astype(dtype)
    _relu_round_trip(x, g)
    _relu_round_trip(x, g, in_place=True)


def test_relu_special_values_and_negative_gradients():
    x = np.array([-0.0, 0.0, -np.inf, np.inf, 1e-45, -1e-45, 3.0, -3.0] * 40, dtype=np.float32)
    g = np.array([-1, 2, -3, -np.inf, 5, -6, -7, -8] * 40, dtype=np.float32)
    _relu_round_trip(x, g)
    _relu_round_trip(x.astype(np.float16), g.astype(np.float16))


def test_relu_stem_size():
    """ReLU after the ResNet-50 stem at batch 32: fp32 [32,64,112,112]."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal((32, 64, 112, 112), dtype=np.float32)
    g = rng.standard_normal((32, 64, 112, 112), dtype=np.float32)
    _relu_round_trip(x, g)


CONFIGS = [
    # planes-shape, H, W, kernel, stride, padding, dilation
    ((2, 3), 112, 112, (3, 3), (2, 2), (1, 1), (1, 1)),
    ((5,), 8, 8, (2, 2), (2, 2), (0, 0), (1, 1)),
    ((3,), 9, 11, (3, 2), (1, 2), (1, 0), (2, 1)),
    ((4,), 7, 5, (1, 1), (1, 1), (0, 0), (1, 1)),
    ((2, 2), 13, 17, (5, 4), (3, 2), (2, 2), (1, 2)),
    ((1,), 16, 16, (16, 16), (1, 1), (0, 0), (1, 1)),
    ((7,), 6, 6, (3, 3), (1, 1), (1, 1), (1, 1)),
    ((1, 1), 1, 1, (1, 1), (1, 1), (0, 0), (1, 1)),
    ((3,), 33, 65, (3, 3), (2, 2), (1, 1), (1, 1)),
    ((2,), 40, 37, (7, 5), (5, 3), (3, 2), (1, 1)),
    ((2,), 29, 31, (4, 6), (7, 6), (2, 3), (3, 2)),
    ((70000,), 4, 4, (2, 2), (2, 2), (0, 0), (1, 1)),
    ((3,), 12, 16, (3, 3), (1, 1), (1, 1), (1, 1)),     # fast path, stride 1
    ((3,), 11, 13, (2, 2), (1, 1), (1, 1), (1, 1)),
    ((3,), 14, 20, (2, 2), (2, 2), (1, 1), (1, 1)),
    ((3,), 15, 19, (3, 3), (2, 2), (0, 0), (1, 1)),
    ((2,), 17, 24, (3, 3), (2, 2), (1, 0), (1, 1)),
    ((5,), 12, 16, (3, 3), (2, 2), (1, 1), (1, 1)),     # two outputs per lane
    ((5,), 9, 4, (3, 3), (2, 2), (1, 1), (1, 1)),
    ((3,), 10, 36, (2, 2), (2, 2), (0, 0), (1, 1)),
    ((3,), 7, 8, (3, 3), (2, 2), (0, 1), (1, 1)),
    ((4,), 11, 24, (3, 3), (2, 2), (1, 1), (1, 1)),     # eight inputs per lane in the backward pass
    ((4,), 6, 32, (2, 2), (2, 2), (0, 0), (1, 1)),
    ((2,), 5, 8, (3, 3), (2, 2), (1, 1), (1, 1)),
    ((3,), 6, 520, (3, 3), (2, 2), (1, 1), (1, 1)),     # flattened rows: longer than a wavefront covers
    ((3,), 4, 264, (2, 2), (2, 2), (0, 0), (1, 1)),
    ((7,), 2, 8, (3, 3), (2, 2), (1, 1), (1, 1)),       # one output row per plane: first and last at once
    ((9,), 10, 24, (3, 3), (2, 2), (1, 1), (1, 1)),     # lanes of one wavefront in several planes
     # more planes than one grid dimension holds
]


def _pool_round_trip(x_np, g_np, H, W, k, s, p, d):
    dev = torch.device("cuda:0")
    x = torch.from_numpy(x_np).to(dev)
    oy, oarg = oracle.maxpool2d_forward(x_np, k, s, p, d)
    nout = oy.size
    ybuf = torch.full((nout + 64,), float("nan"), dtype=x.dtype, device=dev)
    abuf = torch.full((nout + 64,), CANARY, dtype=torch.uint8, device=dev)
    y, arg = B.maxpool2d_forward(x, k, s, p, d, ybuf[:nout].view(oy.shape), abuf[:nout].view(oy.shape))
    torch.cuda.synchronize()
    assert torch.isnan(ybuf[nout:]).all() and (abuf[nout:] == CANARY).all()
    assert np.array_equal(arg.cpu().numpy(), oarg)
    assert _bits_equal(y.cpu().numpy(), oy)
    gy = torch.from_numpy(g_np).to(dev)
    gbuf = torch.full((x_np.size + 64,), float("nan"), dtype=x.dtype, device=dev)
    gx = B.maxpool2d_backward(arg, gy, H, W, k, s, p, d, gbuf[:x_np.size].view(x_np.shape))
    torch.cuda.synchronize()
    assert torch.isnan(gbuf[x_np.size:]).all()
    want = oracle.maxpool2d_backward(oarg, g_np, H, W, k, s, p, d)
    assert _bits_equal(gx.cpu().numpy(), want)


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
@pytest.mark.parametrize("cfg", CONFIGS)
def test_maxpool_configs(cfg, dtype):
    lead, H, W, k, s, p, d = cfg
    rng = np.random.default_rng(H * 100 + W)
    x = rng.standard_normal(lead + (H, W)).astype(dtype)
    OH, OW = oracle.pool2d_output_size(H, W, k, s, p, d)
    assert B.pool2d_output_size(H, W, k, s, p, d) == (OH, OW)
    g = rng.standard_normal(lead + (OH, OW)).astype(dtype)
    _pool_round_trip(x, g, H, W, k, s, p, d)
    # many ties: small integers
    xi = rng.integers(-2, 3, size=lead + (H, W)).astype(dtype)
    _pool_round_trip(xi, g, H, W, k, s, p, d)


def test_maxpool_backward_ignores_positions_outside_the_image():
    x = np.random.default_rng(0).standard_normal((1, 6, 6)).astype(np.float32)
    _, arg = oracle.maxpool2d_forward(x, (3, 3), (2, 2), (1, 1))
    gy = np.ones((1, 3, 3), dtype=np.float32)
    bad = arg.copy()
    bad[0, 0, 0] = 0          # points at the padding
    bad[0, 1, 1] = 200        # outside the window
    gx = B.maxpool2d_backward(torch.from_numpy(bad).cuda(), torch.from_numpy(gy).cuda(), 6, 6, (3, 3), (2, 2), (1, 1))
    good = arg.copy()
    want = oracle.maxpool2d_backward(good, gy, 6, 6, (3, 3), (2, 2), (1, 1))
    got = gx.cpu().numpy()
    assert got.sum() == want.sum() - 2          # exactly the two bad outputs are dropped


def test_maxpool_stem_size():
    """The one max pooling of ResNet-50 at batch 32: fp32 [32,64,112,112], 3x3, stride 2, padding 1."""
    rng = np.random.default_rng(2)
    x = np.maximum(rng.standard_normal((32, 64, 112, 112), dtype=np.float32), 0)   # post-ReLU: many ties at 0
    g = rng.standard_normal((32, 64, 56, 56), dtype=np.float32)
    _pool_round_trip(x, g, 112, 112, (3, 3), (2, 2), (1, 1), (1, 1))


@pytest.mark.parametrize("dtype", [np.float32, np.float16])
def test_maxpool_sees_new_contents_of_the_same_buffers(dtype):
    """The pooling kernels take one column per wavefront through the scalar data path; a second
    call on the same buffers, refilled by another kernel on the same stream, must see the new
    contents (rows longer than a wavefront covers, so that those columns are in use)."""
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(17)
    planes, H, W = 3, 6, 520
    k, s, p = (3, 3), (2, 2), (1, 1)
    OH, OW = B.pool2d_output_size(H, W, k, s, p)
    x = torch.empty((planes, H, W), dtype=NP[dtype], device=dev)
    y = torch.empty((planes, OH, OW), dtype=NP[dtype], device=dev)
    arg = torch.empty((planes, OH, OW), dtype=torch.uint8, device=dev)
    gy = torch.empty((planes, OH, OW), dtype=NP[dtype], device=dev)
    gx = torch.empty((planes, H, W), dtype=NP[dtype], device=dev)
    for round_ in range(3):
        x_np = rng.standard_normal((planes, H, W)).astype(dtype)
        g_np = rng.standard_normal((planes, OH, OW)).astype(dtype)
        staged_x, staged_g = torch.from_numpy(x_np).to(dev), torch.from_numpy(g_np).to(dev)
        x.copy_(staged_x)                       # device-side writes, then the kernels, no synchronisation between
        gy.copy_(staged_g)
        B.maxpool2d_forward(x, k, s, p, (1, 1), y, arg)
        B.maxpool2d_backward(arg, gy, H, W, k, s, p, (1, 1), gx)
        torch.cuda.synchronize()
        oy, oarg = oracle.maxpool2d_forward(x_np, k, s, p)
        assert np.array_equal(arg.cpu().numpy(), oarg), round_
        assert _bits_equal(y.cpu().numpy(), oy), round_
        assert _bits_equal(gx.cpu().numpy(), oracle.maxpool2d_backward(oarg, g_np, H, W, k, s, p)), round_
