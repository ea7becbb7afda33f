"""Activation-compressed layers (Sec. 3.2 Eq. (4), Sec. 5.1): the saved context equals the oracle's
bit for bit, the gradients are the stock backward applied to the dequantized context, the
activation-compressed gradient is unbiased, and a small network trains."""
import numpy as np
import pytest
import torch
import torch.nn as nn
import torch.nn.functional as F

import oracle
from paper_2104_14129_amd import binding as B
from paper_2104_14129_amd import layers as L

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _reset_config():
    saved = L.QConfig(**vars(L.config))
    yield
    for k, v in vars(saved).items():
        setattr(L.config, k, v)


def _context_matches_oracle(x, c):
    """Recompute the context on the CPU from what the device decided (widths) and compare."""
    x_np = x.detach().cpu().numpy().reshape(c.N, c.D)
    bits = c.bits.cpu().numpy()
    return x_np, bits


@pytest.mark.parametrize("mixed", [False, True])
@pytest.mark.parametrize("shape", [(8, 3, 16, 16), (6, 700), (4, 5, 64)])
def test_saved_context_equals_the_oracle(shape, mixed):
    torch.manual_seed(0)
    x = (torch.randn(shape, device=DEV) * torch.exp(torch.randn(shape[0], *([1] * (len(shape) - 1)), device=DEV))).contiguous()
    L.config.mixed, L.config.bits, L.config.seed = mixed, 2.0 if not mixed else 2.5, 99
    import itertools
    L._tags = itertools.count(41)
    c = L.compress(x)
    torch.cuda.synchronize()
    x_np = x.cpu().numpy().reshape(c.N, c.D)
    bits = c.bits.cpu().numpy()
    if mixed:
        gmin, grange = oracle.group_stats(x_np)
        w = B.sample_sensitivity(torch.from_numpy(grange).to(DEV)).cpu().numpy()
        want_bits = oracle.allocate_bits(w, np.full(c.N, c.D, dtype=np.int64), int(2.5 * c.N * c.D))
        assert np.array_equal(bits, want_bits) and len(set(bits)) > 1
    else:
        assert np.all(bits == 2)
    opacked, oheader, ooff = oracle.quantize_pack(x_np, bits, 99, 41, noise_bits=16)
    assert np.array_equal(c.offsets.cpu().numpy().view(np.uint64), ooff)
    assert np.array_equal(c.packed[:opacked.size].cpu().numpy(), opacked)
    assert np.array_equal(c.header.cpu().numpy().view(np.uint32), oheader.reshape(-1).view(np.uint32))
    want = oracle.unpack_dequantize(opacked, oheader, bits, ooff, c.N, c.D)
    got = L.decompress(c).cpu().numpy().reshape(c.N, c.D)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # compression: 2 - 2.5 code bits + 0.25 header bits per element against 32
    if x.numel() >= 4000:
        assert c.nbytes() < x.numel() * 4 / 6


@pytest.mark.parametrize("shape", [(4, 16, 16, 16), (3, 2304)])
def test_saved_context_of_a_binary16_activation_equals_the_oracle(shape):
    """Mixed-precision training (Sec. 6.1) saves binary16 activations: the context is computed from
    the widened values and decompresses to binary16, both as the oracle has them."""
    torch.manual_seed(1)
    x = (torch.randn(shape, device=DEV) * 3).to(torch.float16).contiguous()
    L.config.mixed, L.config.bits, L.config.seed = False, 4.0, 7
    import itertools
    L._tags = itertools.count(5)
    c = L.compress(x)
    torch.cuda.synchronize()
    x_np = x.cpu().numpy().reshape(c.N, c.D)
    bits = c.bits.cpu().numpy()
    assert c.dtype == torch.float16 and np.all(bits == 4)
    opacked, oheader, ooff = oracle.quantize_pack(x_np, bits, 7, 5, noise_bits=16)
    assert np.array_equal(c.packed[:opacked.size].cpu().numpy(), opacked)
    assert np.array_equal(c.header.cpu().numpy().view(np.uint32), oheader.reshape(-1).view(np.uint32))
    want = oracle.unpack_dequantize(opacked, oheader, bits, ooff, c.N, c.D, out_dtype=np.float16)
    got = L.decompress(c)
    assert got.dtype == torch.float16 and tuple(got.shape) == tuple(shape)
    assert np.array_equal(got.cpu().numpy().reshape(c.N, c.D).view(np.uint16), want.view(np.uint16))


def _dequantized_like(layer_input_hook):
    return layer_input_hook


def test_linear_gradients_are_the_stock_backward_on_the_dequantized_context():
    torch.manual_seed(1)
    x = torch.randn(16, 300, device=DEV, requires_grad=True)
    lin = L.QLinear(300, 40).to(DEV)
    gy = torch.randn(16, 40, device=DEV)
    import itertools
    L._tags = itertools.count(7)
    L.config.mixed, L.config.bits, L.config.seed = False, 2, 5
    y = lin(x)
    assert torch.equal(y, F.linear(x, lin.weight, lin.bias))          # forward unchanged
    y.backward(gy)
    x_np = x.detach().cpu().numpy()
    bits = np.full(16, 2, dtype=np.uint8)
    opacked, oheader, ooff = oracle.quantize_pack(x_np, bits, 5, 7, noise_bits=16)
    xhat = oracle.unpack_dequantize(opacked, oheader, bits, ooff, 16, 300).astype(np.float64)
    want_w = gy.cpu().numpy().astype(np.float64).T @ xhat
    assert np.allclose(lin.weight.grad.cpu().numpy(), want_w, rtol=1e-4, atol=1e-4)
    assert np.allclose(lin.bias.grad.cpu().numpy(), gy.sum(0).cpu().numpy(), rtol=1e-5, atol=1e-5)
    assert torch.allclose(x.grad, gy @ lin.weight.detach(), rtol=1e-5, atol=1e-5)   # does not involve the context
    # and it differs from the exact gradient (the context really was quantized)
    exact_w = gy.cpu().numpy().astype(np.float64).T @ x_np.astype(np.float64)
    assert not np.allclose(want_w, exact_w, rtol=1e-3, atol=1e-3)


def _stock_grads(make_out, params, x_like):
    out = make_out(x_like)
    return out


def test_conv_and_batchnorm_backward_use_the_dequantized_context():
    torch.manual_seed(2)
    x = torch.randn(4, 8, 12, 12, device=DEV, requires_grad=True)
    conv = L.QConv2d(8, 6, 3, stride=2, padding=1).to(DEV)
    bn = L.QBatchNorm2d(6).to(DEV)
    import itertools
    L.config.mixed, L.config.bits, L.config.seed = False, 4, 3
    L._tags = itertools.count(100)
    h = conv(x)
    y = bn(h)
    gy = torch.randn_like(y)
    y.backward(gy)
    got = [p.grad.clone() for p in (conv.weight, conv.bias, bn.weight, bn.bias)] + [x.grad.clone()]

    # reference: the same contexts rebuilt by hand (tags 100 and 101), stock autograd on them
    L._tags = itertools.count(100)
    xhat = L.decompress(L.compress(x.detach()))
    hhat = L.decompress(L.compress(h.detach()))
    # conv: grad_w from (gh, xhat); grad_x from (gh, w).  bn: grads from (gy, hhat) with the batch statistics of h.
    mean, var = h.detach().mean((0, 2, 3)), h.detach().var((0, 2, 3), unbiased=False)
    invstd = torch.rsqrt(var + bn.eps)
    gh, gbw, gbb = torch.ops.aten.native_batch_norm_backward(gy, hhat, bn.weight.detach(), None, None, mean, invstd,
                                                             True, bn.eps, [True, True, True])
    gx, gw, gb = torch.ops.aten.convolution_backward(gh, xhat, conv.weight.detach(), [6], [2, 2], [1, 1], [1, 1], False,
                                                     [0, 0], 1, [True, True, True])
    for a, b in zip(got, [gw, gb, gbw, gbb, gx]):
        assert torch.allclose(a, b, rtol=1e-4, atol=1e-5)
    assert torch.allclose(h, F.conv2d(x, conv.weight, conv.bias, 2, 1))


def test_relu_and_maxpool_modules_are_exact():
    torch.manual_seed(3)
    x = torch.randn(4, 8, 30, 30, device=DEV, requires_grad=True)
    x2 = x.detach().clone().requires_grad_(True)
    q = nn.Sequential(L.QReLU(), L.QMaxPool2d(3, 2, 1))
    s = nn.Sequential(nn.ReLU(), nn.MaxPool2d(3, 2, 1))
    yq, ys = q(x), s(x2)
    assert torch.equal(yq, ys)
    g = torch.randn_like(yq)
    yq.backward(g)
    ys.backward(g)
    assert torch.allclose(x.grad, x2.grad, rtol=0, atol=1e-6)     # sums of up to four terms: order may differ
    assert torch.equal(x.grad != 0, x2.grad != 0)


def test_activation_compressed_gradient_is_unbiased():
    torch.manual_seed(4)
    x = torch.randn(32, 512, device=DEV)
    lin = L.QLinear(512, 16, bias=False).to(DEV)
    gy = torch.randn(32, 16, device=DEV)
    L.config.mixed, L.config.bits = True, 2.0
    exact = gy.t() @ x
    S = 300
    acc = torch.zeros_like(exact)
    acc2 = torch.zeros_like(exact)
    for s in range(S):
        lin.weight.grad = None
        lin(x).backward(gy)
        acc += lin.weight.grad
        acc2 += lin.weight.grad ** 2
    mean = acc / S
    var = (acc2 / S - mean ** 2).clamp_min(1e-12)
    z = (mean - exact) / (var / S).sqrt()
    assert z.abs().max().item() < 5.5
    assert (var.sqrt() / exact.abs().mean()).mean().item() > 1e-3      # there is noise to average


def test_swapping_keeps_the_context_on_the_host_and_the_gradients_unchanged():
    import itertools
    torch.manual_seed(5)
    x = torch.randn(8, 4, 16, 16, device=DEV, requires_grad=True)
    conv = L.QConv2d(4, 4, 3, padding=1).to(DEV)
    gy = torch.randn(8, 4, 16, 16, device=DEV)
    grads, contexts = [], []
    for swap in (False, True):
        L.config.mixed, L.config.bits, L.config.swap, L.config.seed = True, 3.0, swap, 11
        L._tags = itertools.count(500)
        conv.weight.grad = None
        c = L.compress(x.detach())
        assert (c.packed is None) == swap and (c.host is not None) == swap
        if swap:
            assert c.host[0].is_pinned() and not c.host[0].is_cuda
        contexts.append(L.decompress(c).clone())
        L._tags = itertools.count(500)
        conv(x).backward(gy)
        grads.append(conv.weight.grad.clone())
    assert torch.equal(contexts[0], contexts[1])                    # the same context, bit for bit
    assert torch.allclose(grads[0], grads[1], rtol=1e-5, atol=1e-4)  # the library's weight gradient may reorder sums


def test_a_small_network_trains_with_compressed_activations():
    def make():
        torch.manual_seed(6)
        return nn.Sequential(nn.Conv2d(3, 16, 3, padding=1), nn.BatchNorm2d(16), nn.ReLU(), nn.MaxPool2d(2, 2),
                             nn.Conv2d(16, 32, 3, padding=1), nn.BatchNorm2d(32), nn.ReLU(), nn.MaxPool2d(2, 2),
                             nn.Flatten(), nn.Linear(32 * 4 * 4, 10)).to(DEV)

    gen = torch.Generator(device=DEV).manual_seed(7)
    proto = torch.randn(10, 3, 16, 16, device=DEV, generator=gen)
    labels = torch.randint(0, 10, (256,), device=DEV, generator=gen)
    data = proto[labels] + 0.5 * torch.randn(256, 3, 16, 16, device=DEV, generator=gen)

    def train(model):
        opt = torch.optim.SGD(model.parameters(), lr=0.05, momentum=0.9)
        losses = []
        for step in range(40):
            idx = torch.arange(64, device=DEV) + 64 * (step % 4)
            loss = F.cross_entropy(model(data[idx]), labels[idx])
            opt.zero_grad()
            loss.backward()
            opt.step()
            losses.append(loss.item())
        return losses

    stock = train(make())
    L.set_optimization_level("L3", bits=2.0)
    q = L.convert(make())
    assert isinstance(q[0], L.QConv2d) and isinstance(q[2], L.QReLU) and isinstance(q[9], L.QLinear)
    compressed = train(q)
    assert compressed[0] == pytest.approx(stock[0], rel=1e-4)       # same forward at the first step
    assert compressed[-1] < 0.3 * compressed[0]                      # it learns
    assert compressed[-1] < stock[-1] + 0.3                          # about as well as full precision


def test_a_retained_graph_can_be_walked_twice():
    """The compressed context is handed to autograd, so it lives as long as the graph: a second
    backward pass over a retained graph dequantizes the same context and gives the same gradients."""
    torch.manual_seed(3)
    L.config.mixed, L.config.bits = False, 4.0
    net = nn.Sequential(L.QConv2d(3, 8, 3, padding=1), L.QBatchNorm2d(8), L.QReLU(), L.QMaxPool2d(2),
                        nn.Flatten(), L.QLinear(8 * 8 * 8, 5)).to(DEV)
    x = torch.randn(4, 3, 16, 16, device=DEV, requires_grad=True)
    loss = net(x).square().sum()
    first = torch.autograd.grad(loss, [x, *net.parameters()], retain_graph=True)
    second = torch.autograd.grad(loss, [x, *net.parameters()])
    for a, b in zip(first, second):       # the stock convolution backward may add in a different order
        assert torch.allclose(a, b, rtol=1e-4, atol=1e-5 * float(a.abs().max()))


def test_layers_run_under_autocast():
    """Under autocast the layer's output, and so the incoming gradient, is binary16 while the saved
    input and the weights are binary32: the backward computes in the gradient's type and returns
    gradients of the operands' types, as the stock layers do."""
    torch.manual_seed(4)
    L.config.mixed, L.config.bits = False, 8.0
    stock = nn.Sequential(nn.Conv2d(3, 8, 3, padding=1), nn.ReLU(), nn.Flatten(), nn.Linear(8 * 12 * 12, 6)).to(DEV)
    ours = nn.Sequential(L.QConv2d(3, 8, 3, padding=1), L.QReLU(), nn.Flatten(), L.QLinear(8 * 12 * 12, 6)).to(DEV)
    ours.load_state_dict(stock.state_dict())
    x = torch.randn(5, 3, 12, 12, device=DEV)
    grads = []
    for net in (stock, ours):
        xin = x.clone().requires_grad_(True)
        with torch.autocast("cuda", dtype=torch.float16):
            y = net(xin)
            assert y.dtype == torch.float16
            loss = y.float().square().mean()
        loss.backward()
        assert xin.grad.dtype == torch.float32 and all(p.grad.dtype == torch.float32 for p in net.parameters())
        grads.append([xin.grad.clone()] + [p.grad.clone() for p in net.parameters()])
    # 8-bit contexts of binary16-rounded activations: the gradients agree to binary16 accuracy
    for a, b in zip(*grads):
        assert torch.allclose(a, b, rtol=5e-2, atol=5e-3 * float(a.abs().max()))
