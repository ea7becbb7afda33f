"""The seeded input generators produce the workloads the measurements are quoted on: shapes,
element types, width multisets, value laws and structure, identically on every call."""
import numpy as np

from paper_2104_14129_amd import synth


def test_tiny_workload():
    wl = synth.tiny()
    x = synth.make_input(wl)
    assert x.shape == (4, 64, 8, 8) and x.dtype == np.float32 and list(wl.bits) == [2, 2, 2, 2]
    assert abs(float(x.mean())) < 0.05 and abs(float(x.std()) - 1.0) < 0.05     # N(0, 1)
    assert np.array_equal(x, synth.make_input(synth.tiny()))                    # the same tensor on every call


def test_stage1_workload_widths_and_values():
    wl = synth.r50_stage1()
    assert wl.shape == (128, 256, 56, 56) and wl.dtype == "f32" and wl.D == 256 * 56 * 56 and wl.ng == 3136
    counts = {int(b): int((wl.bits == b).sum()) for b in np.unique(wl.bits)}
    assert counts == {1: 80, 2: 24, 4: 16, 8: 8} and float(wl.bits.mean()) == 2.0
    assert np.array_equal(wl.bits, synth.r50_stage1().bits)                     # the seeded order of the widths
    small = synth.r50_stage1(N=16)
    assert {int(b): int((small.bits == b).sum()) for b in np.unique(small.bits)} == {1: 10, 2: 3, 4: 2, 8: 1}
    x = synth.make_input(small)
    assert x.shape == (16, 256, 56, 56) and x.min() == 0.0                      # max(0, N(0, 1))
    zeros = float((x == 0).mean())
    assert 0.49 < zeros < 0.51
    pos = x[x > 0]
    assert abs(float(pos.mean()) - 0.7979) < 0.01                               # mean of a half-normal: sqrt(2 / pi)


def test_stem_workload_has_dead_planes_in_binary16():
    wl = synth.r50_stem_f16(N=8)
    x = synth.make_input(wl)
    assert x.shape == (8, 64, 112, 112) and x.dtype == np.float16 and np.all(wl.bits == 2)
    dead = (x.reshape(8, 64, -1) == 0).all(axis=2)
    assert 0.04 < float(dead.mean()) < 0.17                                     # 10 % of the (sample, channel) planes
    live = x.reshape(8, 64, -1)[~dead].astype(np.float32)
    assert abs(float(live[live > 0].mean()) - 1.5 * 0.7979) < 0.02              # sigma = 1.5
    assert synth.r50_stem_f16().shape == (256, 64, 112, 112)


def test_fpn_workload_channel_scales_and_width_sets():
    for variant, counts in ((0, {1: 4, 2: 2, 4: 2}), (1, {1: 6, 2: 1, 8: 1})):
        wl = synth.fpn(variant)
        assert wl.shape == (8, 256, 200, 304) and wl.dtype == "f32"
        assert {int(b): int((wl.bits == b).sum()) for b in np.unique(wl.bits)} == counts
        assert float(wl.bits.mean()) == 2.0
    wl = synth.fpn(0, H=20, W=32)                                               # the same law on a small plane
    x = synth.make_input(wl)
    scale = np.abs(x).mean(axis=(0, 2, 3))                                      # E|Laplace(0, s)| = s
    assert scale.min() > 0.008 and scale.max() < 12.5 and scale.max() / scale.min() > 100
    assert abs(float(np.median(x))) < 0.01
    kurt = float(((x / scale[None, :, None, None]) ** 4).mean())                # heavy tails: E[(x/s)^4] = 24
    assert 18 < kurt < 30


def test_sweep_shapes_are_the_53_convolution_inputs_of_resnet50():
    shapes = synth.resnet50_conv_input_shapes()
    assert len(shapes) == 53 and shapes[0] == (3, 224, 224) and shapes[1] == (64, 56, 56) and shapes[-1] == (512, 7, 7)
    assert sum(c * h * w for c, h, w in shapes) == 10_662_400
    assert max(c * h * w for c, h, w in shapes) == 256 * 56 * 56 and min(c * h * w for c, h, w in shapes) == 512 * 7 * 7
    assert all((c * h * w) % 256 == 0 for c, h, w in shapes)                    # full groups throughout
    w = synth.lognormal_sensitivities(53 * 256, seed=9)
    assert w.dtype == np.float32 and w.shape == (13568,) and w.min() > 0
    assert abs(float(np.log(w).mean())) < 0.03 and abs(float(np.log(w).std()) - 1.0) < 0.03
    assert np.array_equal(w, synth.lognormal_sensitivities(53 * 256, seed=9))
