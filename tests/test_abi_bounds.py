"""Host-side argument checks of the C ABI at their exact limits, one violated condition per call
with every other argument valid, so that a check that was weakened, shadowed by a later one or
given the wrong constant shows.  Every call here must be refused before anything is launched
(no GPU needed; the pointers are never dereferenced).  The limits come from include/actq.h."""
import ctypes

import numpy as np
import pytest

from paper_2104_14129_amd import binding as B

FAKE = 0x10000       # non-null, 4096-byte aligned, never dereferenced
HUGE = 1 << 62       # a capacity that no size check can object to
E = B.ACTQ_EINVAL


def _refused(fn, ok, idx, bad):
    args = list(ok)
    args[idx] = bad
    rc = fn(*args)
    assert rc == E, (fn.__name__, idx, bad, rc, B.last_error())
    assert B.last_error()


# x, dt, N, D, G, gmin, grange, stream
GROUP_STATS_OK = [FAKE, 0, 4, 512, 256, FAKE, FAKE, None]


@pytest.mark.parametrize("idx,bad", [
    (2, 1 << 32), (2, 0), (2, -1),                    # N in [1, 2^32)
    (3, 1 << 34), (3, 0), (3, -256),                  # D in [1, 2^34)
    (4, 255), (4, 257), (4, 0), (4, 512),             # G = 256 only
    (1, 2), (1, -1),                                  # dtype
    (0, FAKE + 8), (0, FAKE + 4), (0, FAKE + 1),      # x: 16 bytes
    (5, FAKE + 2), (5, FAKE + 1), (5, FAKE + 3),      # gmin: 4 bytes
    (6, FAKE + 2), (6, FAKE + 1), (6, FAKE + 3),      # grange: 4 bytes
    (0, None), (5, None), (6, None),
])
def test_group_stats_limits(idx, bad):
    _refused(B.lib().actq_group_stats, GROUP_STATS_OK, idx, bad)


def test_element_count_that_overflows_the_index_arithmetic():
    L = B.lib()
    # N * ng * 256 must not exceed 2^62: N = 2^31, D = 2^33 - 256 gives 2^64 - 2^39
    assert L.actq_group_stats(FAKE, 0, 1 << 31, (1 << 33) - 256, 256, FAKE, FAKE, None) == E
    assert "too large" in B.last_error()
    # just above the limit: ng = 2^20, N = 2^34 / ... is capped by N < 2^32 first, so use ng = 2^25: limit N = 2^29
    assert L.actq_group_stats(FAKE, 0, (1 << 29) + 1, 1 << 33, 256, FAKE, FAKE, None) == E
    assert "too large" in B.last_error()


# x, dt, N, D, G, bits, offsets, seed, tag, noise_bits, packed, capacity, header, hf, stream
QUANTIZE_OK = [FAKE, 0, 2, 512, 256, FAKE, FAKE, 1, 0, 16, FAKE, HUGE, FAKE, 0, None]


@pytest.mark.parametrize("idx,bad", [
    (9, 0), (9, 8), (9, 15), (9, 17), (9, 23), (9, 25), (9, 32), (9, -16), (9, 40),     # noise_bits in {16, 24}
    (13, 3), (13, -1),                                                                   # header format
    (1, 2),
    (2, 1 << 32), (3, 1 << 34),
    (0, FAKE + 8), (10, FAKE + 8), (10, FAKE + 4), (12, FAKE + 4), (12, FAKE + 2), (6, FAKE + 4), (6, FAKE + 2),
    (5, FAKE + 2), (5, FAKE + 1), (5, FAKE + 3),
    (11, 2 * 2 * 32 - 1), (11, 0),                   # capacity below one bit per element: N * ng * 32 bytes
])
def test_quantize_pack_limits(idx, bad):
    _refused(B.lib().actq_quantize_pack, QUANTIZE_OK, idx, bad)


def test_quantize_pack_capacity_counts_the_ragged_last_group():
    # D = 257 has two groups per sample: one bit per element of both is 2 * 32 bytes per sample
    ok = list(QUANTIZE_OK)
    ok[3] = 257
    _refused(B.lib().actq_quantize_pack, ok, 11, 2 * 2 * 32 - 1)
    ok[3] = 3 * 256 + 1
    _refused(B.lib().actq_quantize_pack, ok, 11, 2 * 4 * 32 - 1)


# packed, capacity, header, hf, bits, offsets, N, D, G, out, out_dt, stream
DEQUANTIZE_OK = [FAKE, HUGE, FAKE, 0, FAKE, FAKE, 2, 512, 256, FAKE, 0, None]


@pytest.mark.parametrize("idx,bad", [
    (3, 3), (10, 2), (6, 1 << 32), (7, 1 << 34), (8, 128),
    (9, FAKE + 8), (0, FAKE + 8), (2, FAKE + 4), (5, FAKE + 4), (4, FAKE + 2), (4, FAKE + 1),
])
def test_unpack_dequantize_limits(idx, bad):
    _refused(B.lib().actq_unpack_dequantize, DEQUANTIZE_OK, idx, bad)


# grange, N, ng, G, grad2, w, stream
SENSITIVITY_OK = [FAKE, 4, 16, 256, FAKE, FAKE, None]


@pytest.mark.parametrize("idx,bad", [
    (1, 1 << 32), (1, 0), (1, -3), (2, 1 << 32), (2, 0), (2, -1), (3, 0), (3, -256),
    (0, FAKE + 2), (0, FAKE + 1), (4, FAKE + 2), (4, FAKE + 1), (4, FAKE + 3), (5, FAKE + 2), (5, FAKE + 1),
    (0, None), (5, None),
])
def test_sample_sensitivity_limits(idx, bad):
    _refused(B.lib().actq_sample_sensitivity, SENSITIVITY_OK, idx, bad)


# w, D_items, D, M, G, budget, widths, bits, offsets, result, stream
ALLOCATE_DEVICE_OK = [FAKE, None, 4096, 8, 256, 1 << 16, B.ACTQ_WIDTHS_POW2, FAKE, FAKE, FAKE, None]


@pytest.mark.parametrize("idx,bad", [
    (3, 1 << 31), (3, 0), (3, -1),                    # M in [1, 2^31)
    (2, 1 << 34), (2, 0), (2, -4096),                 # D in [1, 2^34) when there are no per-item sizes
    (5, -1),
    (6, 0), (6, 1), (6, 1 << 9), (6, B.ACTQ_WIDTHS_POW2 | 1),
    (4, 255), (4, 0),
    (0, FAKE + 2), (0, FAKE + 1), (8, FAKE + 4), (8, FAKE + 2), (9, FAKE + 4), (9, FAKE + 1),
])
def test_allocate_bits_device_limits(idx, bad):
    _refused(B.lib().actq_allocate_bits_device, ALLOCATE_DEVICE_OK, idx, bad)


def test_allocate_bits_device_total_bits_must_fit_63_bits():
    ok = list(ALLOCATE_DEVICE_OK)
    ok[2], ok[3] = 1 << 33, 1 << 27                   # D * M * 8 = 2^63 exactly
    assert B.lib().actq_allocate_bits_device(*ok) == E
    ok = list(ALLOCATE_DEVICE_OK)
    ok[1] = FAKE + 4                                  # per-item sizes: 8-byte aligned
    assert B.lib().actq_allocate_bits_device(*ok) == E


def test_allocate_bits_host_budget_limits():
    """A budget of zero is a valid argument (the answer is 'infeasible', with every width at the
    narrowest); budgets that are met exactly stop the greedy exactly there."""
    w = np.array([1.0, 2.0, 3.0], dtype=np.float32)
    D = np.full(3, 256, dtype=np.int64)
    with pytest.raises(B.ActqError) as e:
        B.allocate_bits(w, D, 0)
    assert e.value.code == B.ACTQ_EINFEASIBLE
    assert list(B.allocate_bits(w, D, 8 * 3 * 256)) == [8, 8, 8]            # exactly loose: nothing moves
    assert list(B.allocate_bits(w, D, 8 * 3 * 256 - 1)) == [4, 8, 8]        # one bit short: the cheapest move
    assert list(B.allocate_bits(w, D, (4 + 8 + 8) * 256)) == [4, 8, 8]      # met exactly: no further move
    assert list(B.allocate_bits(w, D, 3 * 256)) == [1, 1, 1]                # exactly the narrowest everywhere
    one = B.allocate_bits(np.ones(1, dtype=np.float32), np.full(1, 256, dtype=np.int64), 4 * 256)
    assert list(one) == [4]


# x, dt, n, zr, stream
TENSOR_STATS_OK = [FAKE, 0, 1000, FAKE, None]


@pytest.mark.parametrize("idx,bad", [(2, 1 << 40), (2, 0), (2, -1), (0, FAKE + 8), (0, FAKE + 4), (3, FAKE + 4),
                                     (3, FAKE + 2), (1, 2)])
def test_tensor_stats_limits(idx, bad):
    _refused(B.lib().actq_tensor_stats, TENSOR_STATS_OK, idx, bad)


# x, dt, n, y, mask, stream
RELU_OK = [FAKE, 0, 1000, FAKE, FAKE, None]


@pytest.mark.parametrize("idx,bad", [(2, 1 << 40), (2, 0), (0, FAKE + 8), (3, FAKE + 8), (4, FAKE + 8), (0, FAKE + 4),
                                     (3, FAKE + 2), (4, FAKE + 1), (1, 2)])
def test_relu_limits(idx, bad):
    _refused(B.lib().actq_relu_forward, RELU_OK, idx, bad)
    # relu_backward: mask, grad_y, dt, n, grad_x, stream -- the same checks in its own argument order
    back = {0: 1, 1: 2, 2: 3, 3: 4, 4: 0}
    _refused(B.lib().actq_relu_backward, [FAKE, FAKE, 0, 1000, FAKE, None], back[idx], bad)


# ----------------------------------------------------------------------------- pooling geometry

def _size(H=8, W=8, kh=3, kw=3, sh=2, sw=2, ph=1, pw=1, dh=1, dw=1):
    oh, ow = ctypes.c_int32(-7), ctypes.c_int32(-7)
    rc = B.lib().actq_pool2d_output_size(H, W, kh, kw, sh, sw, ph, pw, dh, dw, ctypes.addressof(oh), ctypes.addressof(ow))
    return rc, oh.value, ow.value


@pytest.mark.parametrize("change", [
    dict(H=0), dict(W=0), dict(H=-1), dict(kh=0), dict(kw=0), dict(sh=0), dict(sw=0), dict(dh=0), dict(dw=0),
    dict(ph=-1), dict(pw=-1), dict(ph=2), dict(pw=2),                         # padding above half the window
    dict(kh=257, kw=1, H=300, ph=0), dict(kh=1, kw=257, W=300, pw=0), dict(kh=17, kw=16, H=40, W=40),   # more than 256 positions
    dict(H=2, ph=0, kh=3), dict(W=2, pw=0, kw=3),                              # the window does not fit
    dict(kh=2, ph=0, dh=1 << 20, H=1 << 21), dict(kw=2, pw=0, dw=1 << 20, W=1 << 21),                 # extent above 2^20
    dict(H=(1 << 24) + 1), dict(W=(1 << 24) + 1), dict(sh=(1 << 20) + 1), dict(sw=(1 << 20) + 1),
    dict(H=1 << 16, W=1 << 15),                                                # 2^31 locations
])
def test_pooling_geometry_refused(change):
    assert _size() == (0, 4, 4)
    rc, oh, ow = _size(**change)
    assert rc == E and (oh, ow) == (-7, -7), change


def test_pooling_geometry_at_its_limits():
    assert _size(kh=2, kw=2, ph=1, pw=1) == (0, 5, 5)                          # padding of exactly half the window
    assert _size(kh=16, kw=16, ph=0, pw=0, H=16, W=17, sh=1, sw=1) == (0, 1, 2)    # 256 positions
    assert _size(kh=256, kw=1, ph=0, pw=0, H=256, W=3, sh=1, sw=1) == (0, 1, 3)
    assert _size(H=1, W=1) == (0, 1, 1)                                        # the window just fits the padded input
    assert _size(kh=2, ph=0, dh=(1 << 20) - 1, H=1 << 20, W=8) == (0, 1, 4)    # extent of exactly 2^20
    assert _size(H=1 << 24, W=8, kh=1, kw=1, ph=0, pw=0, sh=1 << 20, sw=1) == (0, 16, 8)
    assert _size(H=(1 << 15) - 1, W=1 << 16, kh=1, kw=1, ph=0, pw=0, sh=1, sw=1) == (0, (1 << 15) - 1, 1 << 16)
    rc, _, _ = _size(H=(1 << 15) - 1, W=(1 << 16) - 2)                         # with padding: (2^15 + 1) * 2^16 > 2^31
    assert rc == E


# x, dt, planes, H, W, kh, kw, sh, sw, ph, pw, dh, dw, y, argmax, stream
POOL_FORWARD_OK = [FAKE, 0, 6, 8, 8, 3, 3, 2, 2, 1, 1, 1, 1, FAKE, FAKE, None]


@pytest.mark.parametrize("idx,bad", [(2, 0), (2, -1), (2, (1 << 40) // 64), (0, FAKE + 2), (0, FAKE + 1), (13, FAKE + 2),
                                     (13, FAKE + 3), (1, 2), (0, None), (13, None), (14, None)])
def test_maxpool_call_limits(idx, bad):
    _refused(B.lib().actq_maxpool2d_forward, POOL_FORWARD_OK, idx, bad)
    # backward: argmax, grad_y, dt, planes, H, W, kh..dw, grad_x, stream
    ok = [FAKE, FAKE, 0, 6, 8, 8, 3, 3, 2, 2, 1, 1, 1, 1, FAKE, None]
    back = {0: 1, 1: 2, 2: 3, 13: 14, 14: 0}
    _refused(B.lib().actq_maxpool2d_backward, ok, back[idx], bad)


def test_half_precision_tensors_may_be_two_byte_aligned_but_not_odd():
    ok = list(POOL_FORWARD_OK)
    ok[1] = 1
    _refused(B.lib().actq_maxpool2d_forward, ok, 0, FAKE + 1)
    _refused(B.lib().actq_maxpool2d_forward, ok, 13, FAKE + 1)


# ----------------------------------------------------------------------------- several tensors per call

def _table(n=2, **over):
    t = (B.TensorDesc * n)()
    for slot in t:
        slot.x = slot.out = slot.gmin = slot.grange = slot.header = slot.bits = slot.offsets = FAKE
        slot.D = 512
    for k, v in over.items():
        setattr(t[n - 1], k, v)
    return t


def _stats(t, count=None, dt=0, N=4, G=256):
    return B.lib().actq_group_stats_multi(ctypes.addressof(t), len(t) if count is None else count, dt, N, G, None)


def _quant(t, dt=0, N=4, G=256, nb=16, packed=FAKE, hf=0):
    return B.lib().actq_quantize_pack_multi(ctypes.addressof(t), len(t), dt, N, G, 1, 0, nb, packed, HUGE, hf, None)


def _deq(t, dt=0, N=4, G=256, packed=FAKE, hf=0):
    return B.lib().actq_unpack_dequantize_multi(ctypes.addressof(t), len(t), packed, HUGE, hf, N, G, dt, None)


def test_multi_tensor_limits():
    assert B.MAX_TENSORS_PER_CALL == 40
    assert _stats(_table(41)) == E and _stats(_table(2), count=0) == E and _stats(_table(2), count=-1) == E
    assert _stats(_table(1), N=1 << 32) == E and _stats(_table(1), dt=2) == E and _stats(_table(1), G=128) == E
    for nb in (0, 15, 17, 23, 25):
        assert _quant(_table(), nb=nb) == E, nb
    for k, v in [("D", 255), ("D", 257), ("D", 511), ("D", 0), ("D", -512), ("D", 1 << 34)]:
        assert _stats(_table(**{k: v})) == E, (k, v)
    # one misplaced pointer in the last tensor of the table, everything else valid
    for k, v in [("x", FAKE + 8), ("x", FAKE + 4), ("gmin", FAKE + 2), ("gmin", FAKE + 1), ("grange", FAKE + 2),
                 ("grange", FAKE + 3), ("gmin", None), ("grange", None), ("x", None)]:
        assert _stats(_table(**{k: v})) == E, (k, v)
        assert _stats(_table(1, **{k: v})) == E, (k, v)          # also when it is the first and only tensor
    for k, v in [("x", FAKE + 8), ("header", FAKE + 4), ("header", FAKE + 2), ("bits", FAKE + 2), ("bits", FAKE + 1),
                 ("offsets", FAKE + 4), ("offsets", FAKE + 2), ("header", None), ("bits", None), ("offsets", None)]:
        assert _quant(_table(**{k: v})) == E, (k, v)
        assert _quant(_table(1, **{k: v})) == E, (k, v)
    for k, v in [("out", FAKE + 8), ("out", FAKE + 4), ("header", FAKE + 4), ("bits", FAKE + 2), ("offsets", FAKE + 4),
                 ("out", None)]:
        assert _deq(_table(**{k: v})) == E, (k, v)
        assert _deq(_table(1, **{k: v})) == E, (k, v)
    assert _quant(_table(), packed=FAKE + 8) == E and _deq(_table(), packed=FAKE + 8) == E
    assert _quant(_table(), hf=3) == E and _deq(_table(), hf=-1) == E


# ----------------------------------------------------------------------------- host-only entry points, both sides of a limit

def _header_bytes(N, D, hf=0, G=256):
    out = ctypes.c_uint64(7)
    rc = B.lib().actq_header_bytes(N, D, G, hf, ctypes.addressof(out))
    return rc, out.value


def test_size_limits_on_both_sides_through_the_host_only_calls():
    """actq_header_bytes shares the shape checks of the device calls and launches nothing, so the
    accepted side of every limit can be probed as well."""
    assert _header_bytes(1, 1) == (0, 8)                                     # the smallest tensor
    assert _header_bytes((1 << 32) - 1, 256) == (0, ((1 << 32) - 1) * 8)     # N just below 2^32
    assert _header_bytes(1 << 32, 256)[0] == E
    assert _header_bytes(1, (1 << 34) - 1) == (0, (1 << 26) * 8)             # D just below 2^34
    assert _header_bytes(1, 1 << 34)[0] == E
    # N * ng * 256 <= 2^62: D = 2^33 has 2^25 groups, so N = 2^29 is the last one accepted
    assert _header_bytes(1 << 29, 1 << 33) == (0, (1 << 54) * 8)
    assert _header_bytes((1 << 29) + 1, 1 << 33)[0] == E
    # ... and the ragged last group counts: D = 2^33 + 1 has one group more, which lowers the limit
    limit = (1 << 62) // (((1 << 25) + 1) * 256)
    assert limit < 1 << 29
    assert _header_bytes(limit + 1, (1 << 33) + 1)[0] == E
    assert _header_bytes(limit, (1 << 33) + 1) == (0, limit * ((1 << 25) + 1) * 8)
    # group counts of ragged sizes, in all three header formats
    for D, ng in ((255, 1), (256, 1), (257, 2), (511, 2), (512, 2), (513, 3)):
        assert _header_bytes(3, D, 0) == (0, 3 * ng * 8), D
        assert _header_bytes(3, D, 1) == (0, 3 * ng * 4), D
        assert _header_bytes(3, D, 2) == (0, 8), D


def test_packed_bytes_group_counts_and_optional_outputs():
    for D, ng in ((1, 1), (255, 1), (256, 1), (257, 2), (511, 2), (512, 2), (513, 3)):
        off, total = B.packed_bytes(3, D, [1, 8, 3])
        assert list(off) == [0, ng * 32, ng * 32 * 9] and total == ng * 32 * 12, D
    L = B.lib()
    bits = np.array([2, 4], dtype=np.uint8)
    off = np.full(2, 99, dtype=np.uint64)
    tot = ctypes.c_uint64(99)
    assert L.actq_packed_bytes(2, 512, 256, bits.ctypes.data, None, ctypes.addressof(tot)) == 0 and tot.value == 384
    assert L.actq_packed_bytes(2, 512, 256, bits.ctypes.data, off.ctypes.data, None) == 0 and list(off) == [0, 128]
    assert L.actq_packed_bytes(2, 512, 256, bits.ctypes.data, None, None) == E
    assert L.actq_packed_bytes(2, 512, 256, None, off.ctypes.data, ctypes.addressof(tot)) == E
    for bad in ([0, 2], [2, 0], [9, 2], [2, 9]):                            # an invalid width in any position
        b = np.array(bad, dtype=np.uint8)
        assert L.actq_packed_bytes(2, 512, 256, b.ctypes.data, off.ctypes.data, None) == E, bad


def test_allocate_bits_host_null_arguments_one_at_a_time_and_unit_sizes():
    import oracle
    L = B.lib()
    w = np.array([3.0, 1.0, 2.0], dtype=np.float32)
    D = np.array([1, 1, 1], dtype=np.int64)
    out = np.zeros(3, dtype=np.uint8)
    P = B.ACTQ_WIDTHS_POW2
    assert L.actq_allocate_bits(None, D.ctypes.data, 3, 100, P, out.ctypes.data) == E
    assert L.actq_allocate_bits(w.ctypes.data, None, 3, 100, P, out.ctypes.data) == E
    assert L.actq_allocate_bits(w.ctypes.data, D.ctypes.data, 3, 100, P, None) == E
    # items of one element each are valid
    got = B.allocate_bits(w, D, 14)
    assert list(got) == list(oracle.allocate_bits(w, D, 14)) and int(got.sum()) <= 14
    for bad in (0, -1):
        D2 = D.copy()
        D2[2] = bad
        with pytest.raises(B.ActqError) as e:
            B.allocate_bits(w, D2, 14)
        assert e.value.code == E and "D[2]" in str(e.value)


def test_multi_tensor_errors_name_the_offending_tensor():
    for call in (_stats, _quant, _deq):
        for D in (255, 300, 511):
            assert call(_table(3, D=D)) == E
            assert "tensor 2" in B.last_error() and "multiple" in B.last_error(), (call.__name__, D, B.last_error())


@pytest.mark.parametrize("change", [
    dict(kh=0, ph=0), dict(kw=0, pw=0),                                       # an empty window, no padding to trip over
    dict(H=1, ph=1, kh=2, dh=3), dict(W=1, pw=1, kw=2, dw=3),                 # 1 + 2 * 1 < 4: the dilated window does not fit
    dict(H=1 << 16, W=1 << 15, kh=1, kw=1, ph=0, pw=0),                        # exactly 2^31 locations, unpadded
    dict(H=(1 << 16) - 2, W=(1 << 15) - 2),                                    # exactly 2^31 locations with the padding
    dict(H=0, kh=1, ph=0), dict(W=0, kw=1, pw=0),
])
def test_pooling_geometry_refused_by_one_check_only(change):
    rc, oh, ow = _size(**change)
    assert rc == E and (oh, ow) == (-7, -7), change


def test_pooling_geometry_accepted_at_the_remaining_limits():
    assert _size(W=1 << 24, H=8, kh=1, kw=1, ph=0, pw=0, sh=1, sw=1 << 20) == (0, 8, 16)
    assert _size(kw=2, pw=0, dw=(1 << 20) - 1, W=1 << 20, H=8) == (0, 4, 1)
    assert _size(H=(1 << 16) - 1, W=1 << 15, kh=1, kw=1, ph=0, pw=0, sh=1, sw=1) == (0, (1 << 16) - 1, 1 << 15)
    assert _size(H=(1 << 16) - 3, W=(1 << 15) - 2)[0] == 0                     # (2^16 - 1) * 2^15 padded locations
