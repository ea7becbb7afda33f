"""The C ABI library loads, exports every symbol declared in include/actq.h, and rejects
bad arguments on the host before any launch (no GPU needed: nothing here computes)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2104_14129_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x1000  # a non-null, 16-byte aligned address that is never dereferenced by validation


def test_every_declared_symbol_is_exported():
    header = open(os.path.join(ROOT, "include", "actq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(actq_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.version() >= 200


def test_packed_bytes_and_its_errors():
    off, total = B.packed_bytes(4, 1000, [1, 2, 4, 8])
    assert list(off) == [0, 128, 384, 896] and total == 1920
    off, total = B.packed_bytes(5, 1000, [3, 5, 6, 7, 0 + 1])
    assert list(off) == [0, 384, 1024, 1792, 2688] and total == 2816
    with pytest.raises(B.ActqError) as e:
        B.packed_bytes(2, 512, [2, 9])
    assert e.value.code == B.ACTQ_EINVAL and "bits[1]" in str(e.value)
    L = B.lib()
    bits = np.array([2], dtype=np.uint8)
    tot = ctypes.c_uint64()
    assert L.actq_packed_bytes(1, 512, 128, bits.ctypes.data, None, ctypes.addressof(tot)) == B.ACTQ_EINVAL
    assert "group size" in B.last_error()
    assert L.actq_packed_bytes(0, 512, 256, bits.ctypes.data, None, ctypes.addressof(tot)) == B.ACTQ_EINVAL
    assert L.actq_packed_bytes(1, 512, 256, bits.ctypes.data, None, None) == B.ACTQ_EINVAL
    assert L.actq_packed_bytes(1, 512, 256, None, None, ctypes.addressof(tot)) == B.ACTQ_EINVAL


def test_device_calls_validate_before_launching():
    L = B.lib()
    E = B.ACTQ_EINVAL
    # group_stats
    assert L.actq_group_stats(None, 0, 1, 256, 256, FAKE, FAKE, None) == E
    assert L.actq_group_stats(FAKE, 0, 0, 256, 256, FAKE, FAKE, None) == E
    assert L.actq_group_stats(FAKE, 0, 1, 256, 64, FAKE, FAKE, None) == E
    assert L.actq_group_stats(FAKE, 7, 1, 256, 256, FAKE, FAKE, None) == E
    assert L.actq_group_stats(FAKE + 4, 0, 1, 256, 256, FAKE, FAKE, None) == E
    assert "aligned" in B.last_error()
    # quantize_pack: x, dt, N, D, G, bits, offsets, seed, tag, noise_bits, packed, capacity, header, hf, stream
    ok = [FAKE, 0, 2, 512, 256, FAKE, FAKE, 1, 0, 24, FAKE, 1 << 20, FAKE, 0, None]
    assert L.actq_quantize_pack(*(ok[:2] + [2, 512, 128] + ok[5:])) == E      # sanity: list is well-formed
    for idx, bad in [(0, None), (5, None), (6, None), (10, None), (12, None), (2, -1), (3, 0), (4, 512),
                     (1, 3), (9, 12), (0, FAKE + 2), (10, FAKE + 8), (12, FAKE + 4), (11, 10), (2, 1 << 32),
                     (3, 1 << 34), (13, 3), (5, FAKE + 1)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_quantize_pack(*args) == E, (idx, bad)
        assert B.last_error()
    # unpack_dequantize: packed, capacity, header, hf, bits, offsets, N, D, G, out, out_dt, stream
    ok = [FAKE, 1 << 20, FAKE, 1, FAKE, FAKE, 2, 512, 256, FAKE, 0, None]
    for idx, bad in [(0, None), (2, None), (4, None), (5, None), (9, None), (6, 0), (7, -5), (8, 8), (10, 2),
                     (9, FAKE + 4), (0, FAKE + 1), (3, 7), (4, FAKE + 2)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_unpack_dequantize(*args) == E, (idx, bad)
    # sample_sensitivity: grange, N, ng, G, grad2, w, stream
    ok = [FAKE, 4, 16, 256, None, FAKE, None]
    for idx, bad in [(0, None), (5, None), (1, 0), (2, 0), (3, 0), (0, FAKE + 2), (4, FAKE + 1)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_sample_sensitivity(*args) == E, (idx, bad)
    # header_bytes
    out = ctypes.c_uint64()
    assert L.actq_header_bytes(3, 1000, 256, 0, ctypes.addressof(out)) == 0 and out.value == 3 * 4 * 8
    assert L.actq_header_bytes(3, 1000, 256, 1, ctypes.addressof(out)) == 0 and out.value == 3 * 4 * 4
    assert L.actq_header_bytes(3, 1000, 256, 2, ctypes.addressof(out)) == 0 and out.value == 8
    assert L.actq_header_bytes(3, 1000, 256, 5, ctypes.addressof(out)) == E
    # tensor_stats: x, dt, n, zr, stream
    ok = [FAKE, 0, 1000, FAKE, None]
    for idx, bad in [(0, None), (3, None), (1, 4), (2, 0), (2, 1 << 40), (0, FAKE + 4), (3, FAKE + 4)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_tensor_stats(*args) == E, (idx, bad)
    assert L.actq_header_bytes(3, 1000, 256, 0, None) == E


def test_allocate_bits_errors():
    w = np.ones(3, dtype=np.float32)
    D = np.full(3, 256, dtype=np.int64)
    with pytest.raises(B.ActqError) as e:
        B.allocate_bits(w, D, 3 * 256 - 1)
    assert e.value.code == B.ACTQ_EINFEASIBLE and list(e.value.bits) == [1, 1, 1]
    for bad_w in ([-1, 1, 1], [np.nan, 1, 1], [np.inf, 1, 1]):
        with pytest.raises(B.ActqError) as e:
            B.allocate_bits(np.array(bad_w, dtype=np.float32), D, 10 ** 6)
        assert e.value.code == B.ACTQ_EINVAL
    with pytest.raises(B.ActqError):
        B.allocate_bits(w, np.array([256, 0, 256], dtype=np.int64), 10 ** 6)
    L = B.lib()
    out = np.zeros(3, dtype=np.uint8)
    P = B.ACTQ_WIDTHS_POW2
    assert L.actq_allocate_bits(None, D.ctypes.data, 3, 100, P, out.ctypes.data) == B.ACTQ_EINVAL
    assert L.actq_allocate_bits(w.ctypes.data, D.ctypes.data, 0, 100, P, out.ctypes.data) == B.ACTQ_EINVAL
    assert L.actq_allocate_bits(w.ctypes.data, D.ctypes.data, 3, -1, P, out.ctypes.data) == B.ACTQ_EINVAL
    for mask in (0, 1, 1 << 9, P | 1):
        assert L.actq_allocate_bits(w.ctypes.data, D.ctypes.data, 3, 100, mask, out.ctypes.data) == B.ACTQ_EINVAL
        assert "widths" in B.last_error()
    # device allocator: w, D_items, D, M, G, budget, widths, bits, offsets, result, stream
    ok = [FAKE, None, 4096, 8, 256, 1 << 16, P, FAKE, FAKE, FAKE, None]
    for idx, bad in [(0, None), (7, None), (8, None), (9, None), (3, 0), (3, 1 << 31), (4, 128), (2, 0),
                     (2, 1 << 34), (5, -1), (6, 0), (6, 1), (0, FAKE + 2), (8, FAKE + 4), (9, FAKE + 4),
                     (1, FAKE + 4)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_allocate_bits_device(*args) == B.ACTQ_EINVAL, (idx, bad)
        assert B.last_error()


def test_allocate_bits_matches_the_oracle_bit_for_bit():
    """Host logic of the library against the oracle: identical widths, including ties,
    zero sensitivities, unequal sizes and the infeasible case."""
    import oracle
    rng = np.random.default_rng(0)
    for t in range(300):
        M = int(rng.integers(1, 300))
        w = rng.lognormal(0, 2, M).astype(np.float32)
        if t % 3 == 0:
            w[rng.integers(0, M, M // 3 + 1)] = w[0]       # ties
        if t % 5 == 0:
            w[rng.integers(0, M, M // 4 + 1)] = 0.0        # free items
        D = rng.choice([256, 512, 1024, 25088, 802816], M).astype(np.int64)
        budget = int(rng.uniform(0.9, 8.5) * D.sum())
        widths = [B.ACTQ_WIDTHS_POW2, B.ACTQ_WIDTHS_ALL, int(rng.integers(1, 256)) << 1][t % 3]
        try:
            got, gc = B.allocate_bits(w, D, budget, widths), 0
        except B.ActqError as e:
            got, gc = e.bits, e.code
        try:
            want, wc = oracle.allocate_bits(w, D, budget, widths), 0
        except oracle.OracleError as e:
            want, wc = e.bits, e.code
        assert gc == wc
        assert np.array_equal(got, want), t


def test_allocate_bits_full_sweep_size():
    """M = 53 layers x 256 samples, sizes of the ResNet-50 sweep, 2.0-bit budget."""
    import oracle
    from paper_2104_14129_amd import synth
    shapes = synth.resnet50_conv_input_shapes()
    N = 256
    D = np.repeat(np.array([c * h * w for c, h, w in shapes], dtype=np.int64), N)
    w = synth.lognormal_sensitivities(D.size, seed=5)
    budget = 2 * int(D.sum())
    got = B.allocate_bits(w, D, budget)
    want = oracle.allocate_bits(w, D, budget)
    assert np.array_equal(got, want)
    used = int((got.astype(np.int64) * D).sum())
    assert used <= budget and budget - used < 4 * D.max()
    got = B.allocate_bits(w, D, budget, B.ACTQ_WIDTHS_ALL)
    assert np.array_equal(got, oracle.allocate_bits(w, D, budget, oracle.WIDTHS_ALL))
    used = int((got.astype(np.int64) * D).sum())
    assert used <= budget and budget - used < D.max()


def test_context_calls_validate_before_launching():
    L = B.lib()
    E = B.ACTQ_EINVAL
    assert B.relu_mask_bytes(1) == 32 and B.relu_mask_bytes(256) == 32 and B.relu_mask_bytes(257) == 64
    assert L.actq_relu_mask_bytes(0, FAKE) == E and L.actq_relu_mask_bytes(5, None) == E
    # relu_forward: x, dt, n, y, mask, stream
    ok = [FAKE, 0, 1000, FAKE, FAKE, None]
    for idx, bad in [(0, None), (3, None), (4, None), (1, 5), (2, 0), (2, 1 << 40), (0, FAKE + 4), (3, FAKE + 8), (4, FAKE + 1)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_relu_forward(*args) == E, (idx, bad)
    # relu_backward: mask, grad_y, dt, n, grad_x, stream
    ok = [FAKE, FAKE, 1, 1000, FAKE, None]
    for idx, bad in [(0, None), (1, None), (4, None), (2, 2), (3, -1), (0, FAKE + 2), (1, FAKE + 2)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_relu_backward(*args) == E, (idx, bad)
    # output size
    assert B.pool2d_output_size(112, 112, (3, 3), (2, 2), (1, 1)) == (56, 56)
    assert B.pool2d_output_size(9, 11, (3, 2), (1, 2), (1, 0), (2, 1)) == (7, 5)
    for kw in [dict(kernel=(3, 3), stride=(2, 2), padding=(2, 1)), dict(kernel=(17, 16), stride=(1, 1)),
               dict(kernel=(2, 2), stride=(0, 1)), dict(kernel=(2, 2), stride=(1, 1), dilation=(0, 1)),
               dict(kernel=(5, 5), stride=(1, 1)), dict(kernel=(0, 2), stride=(1, 1)),
               dict(kernel=(2, 2), stride=(1, 1), padding=(-1, 0))]:
        with pytest.raises(B.ActqError):
            B.pool2d_output_size(4, 4, **kw)
    # maxpool2d_forward: x, dt, planes, H, W, kh, kw, sh, sw, ph, pw, dh, dw, y, argmax, stream
    ok = [FAKE, 0, 6, 8, 8, 3, 3, 2, 2, 1, 1, 1, 1, FAKE, FAKE, None]
    for idx, bad in [(0, None), (13, None), (14, None), (1, 9), (2, 0), (2, 1 << 40), (3, 0), (5, 20), (7, 0), (9, 2),
                     (0, FAKE + 2), (13, FAKE + 1)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_maxpool2d_forward(*args) == E, (idx, bad)
        assert B.last_error()
    # maxpool2d_backward: argmax, grad_y, dt, planes, H, W, kh..dw, grad_x, stream
    ok = [FAKE, FAKE, 1, 6, 8, 8, 3, 3, 2, 2, 1, 1, 1, 1, FAKE, None]
    for idx, bad in [(0, None), (1, None), (14, None), (2, 3), (3, -2), (4, 0), (1, FAKE + 1)]:
        args = list(ok)
        args[idx] = bad
        assert L.actq_maxpool2d_backward(*args) == E, (idx, bad)


def test_multi_tensor_calls_validate_before_launching():
    L = B.lib()
    E = B.ACTQ_EINVAL

    def table(n=2, **over):
        t = (B.TensorDesc * n)()
        for slot in t:
            slot.x = slot.out = slot.gmin = slot.grange = slot.header = slot.bits = slot.offsets = FAKE
            slot.D = 512
        for k, v in over.items():
            setattr(t[1 if n > 1 else 0], k, v)
        return t

    def stats(t, count=None, dt=0, N=4, G=256):
        return L.actq_group_stats_multi(ctypes.addressof(t), len(t) if count is None else count, dt, N, G, None)

    def quant(t, dt=0, N=4, G=256, nb=16, packed=FAKE, hf=0):
        return L.actq_quantize_pack_multi(ctypes.addressof(t), len(t), dt, N, G, 1, 0, nb, packed, 1 << 20, hf, None)

    def deq(t, dt=0, N=4, G=256, packed=FAKE, hf=0):
        return L.actq_unpack_dequantize_multi(ctypes.addressof(t), len(t), packed, 1 << 20, hf, N, G, dt, None)

    assert L.actq_group_stats_multi(None, 1, 0, 4, 256, None) == E
    assert stats(table(), count=0) == E and stats(table(41)) == E
    assert stats(table(), dt=3) == E and stats(table(), N=0) == E and stats(table(), G=64) == E
    for k, v in [("D", 500), ("D", 0), ("x", None), ("x", FAKE + 4), ("gmin", None), ("grange", FAKE + 2)]:
        assert stats(table(**{k: v})) == E, (k, v)
        assert "tensor 1" in B.last_error() or "D" in B.last_error() or "positive" in B.last_error()
    assert quant(table(), nb=8) == E and quant(table(), packed=None) == E and quant(table(), packed=FAKE + 8) == E
    assert quant(table(), hf=9) == E
    for k, v in [("D", 300), ("x", None), ("header", None), ("header", FAKE + 4), ("bits", None), ("bits", FAKE + 1),
                 ("offsets", None), ("offsets", FAKE + 4)]:
        assert quant(table(**{k: v})) == E, (k, v)
    assert deq(table(), dt=2) == E and deq(table(), packed=None) == E
    for k, v in [("out", None), ("out", FAKE + 8), ("header", None), ("bits", None), ("offsets", None), ("D", 257)]:
        assert deq(table(**{k: v})) == E, (k, v)


def test_the_loaded_library_was_built_from_the_sources_beside_it():
    """The binary carries a digest of its sources and flags; the binding refuses (or rebuilds) a
    library whose digest differs, so an edited kernel is never tested against a stale binary."""
    from paper_2104_14129_amd import build as lib_build
    assert B.source_hash() == lib_build.source_hash()
    assert B._digest_in_file(B.LIB_PATH) == lib_build.source_hash()
    # a binary with another digest is told apart without loading it
    import tempfile
    blob = open(B.LIB_PATH, "rb").read()
    marker = b"actq-source-digest:"
    at = blob.index(marker) + len(marker)
    other = blob[:at] + (b"0" if blob[at:at + 1] != b"0" else b"1") + blob[at + 1:]
    with tempfile.NamedTemporaryFile(suffix=".so") as f:
        f.write(other)
        f.flush()
        assert B._digest_in_file(f.name) != lib_build.source_hash()
    assert B._digest_in_file("/nonexistent/libactq.so") is None
