"""ctypes binding of libactq's C ABI (include/actq.h): argument marshalling only.

Every function takes torch tensors (device memory and streams are PyTorch's) or numpy
arrays for the host-side calls, checks dtypes / contiguity, and forwards raw pointers.
There is no CPU fallback: if the HIP library cannot be loaded the import of the symbols
fails with an error.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libactq.so")

ACTQ_OK, ACTQ_EINVAL, ACTQ_EINFEASIBLE, ACTQ_EHIP = 0, -1, -2, -3
ACTQ_F32, ACTQ_F16 = 0, 1
G_DEFAULT = 256

ACTQ_HDR_F32, ACTQ_HDR_BF16, ACTQ_HDR_TENSOR = 0, 1, 2
ACTQ_WIDTHS_POW2, ACTQ_WIDTHS_ALL = 0x116, 0x1FE  # allowed-width sets of the allocator (bit b = b bits)

EXPORTS = ("actq_version", "actq_source_hash", "actq_last_error", "actq_packed_bytes", "actq_header_bytes", "actq_group_stats",
           "actq_quantize_pack", "actq_unpack_dequantize", "actq_sample_sensitivity", "actq_allocate_bits",
           "actq_allocate_bits_device", "actq_relu_mask_bytes", "actq_relu_forward", "actq_relu_backward",
           "actq_pool2d_output_size", "actq_maxpool2d_forward", "actq_maxpool2d_backward", "actq_tensor_stats",
           "actq_group_stats_multi", "actq_quantize_pack_multi", "actq_unpack_dequantize_multi")


class ActqError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libactq error {code}: {message}")
        self.code = code


_lib = None


def _digest_in_file(path: str):
    """The source digest baked into a built library, read from the file (nothing is loaded)."""
    marker = b"actq-source-digest:"
    try:
        with open(path, "rb") as f:
            blob = f.read()
    except OSError:
        return None
    at = blob.find(marker)
    if at < 0:
        return None
    end = blob.find(b"\0", at)
    return blob[at + len(marker):end].decode(errors="replace")


def _load_checked() -> ctypes.CDLL:
    """libactq.so, built from exactly the sources beside it: a missing library is built; one whose
    baked-in source digest differs from the sources' is rebuilt when a compiler is there and refused
    otherwise (an edited kernel must never be tested or timed against a stale binary)."""
    from . import build as _build
    want = _build.source_hash()
    have = _digest_in_file(LIB_PATH)
    if have != want:
        try:
            _build.build()
        except Exception as exc:
            if not os.path.exists(LIB_PATH):
                raise
            raise RuntimeError(f"{LIB_PATH} was built from other sources (digest {have}, sources {want}) "
                               f"and cannot be rebuilt here: {exc}") from exc
    L = ctypes.CDLL(LIB_PATH)
    L.actq_source_hash.restype = ctypes.c_char_p
    L.actq_source_hash.argtypes = []
    have = L.actq_source_hash().decode()
    if have != want:
        raise RuntimeError(f"{LIB_PATH} reports source digest {have}, the sources beside it have {want}")
    return L


def source_hash() -> str:
    """Digest baked into the loaded library (equal to the digest of the sources beside it)."""
    return lib().actq_source_hash().decode()


def lib() -> ctypes.CDLL:
    """Loads libactq.so, checked against the sources it sits beside."""
    global _lib
    if _lib is not None:
        return _lib
    L = _load_checked()
    c = ctypes
    vp, i64, i32, u64 = c.c_void_p, c.c_int64, c.c_int32, c.c_uint64
    L.actq_version.restype = c.c_int
    L.actq_version.argtypes = []
    L.actq_last_error.restype = c.c_char_p
    L.actq_last_error.argtypes = []
    L.actq_packed_bytes.restype = c.c_int
    L.actq_packed_bytes.argtypes = [i64, i64, i32, vp, vp, vp]
    L.actq_group_stats.restype = c.c_int
    L.actq_group_stats.argtypes = [vp, c.c_int, i64, i64, i32, vp, vp, vp]
    L.actq_quantize_pack.restype = c.c_int
    L.actq_quantize_pack.argtypes = [vp, c.c_int, i64, i64, i32, vp, vp, u64, u64, i32, vp, u64, vp, c.c_int, vp]
    L.actq_unpack_dequantize.restype = c.c_int
    L.actq_unpack_dequantize.argtypes = [vp, u64, vp, c.c_int, vp, vp, i64, i64, i32, vp, c.c_int, vp]
    L.actq_header_bytes.restype = c.c_int
    L.actq_header_bytes.argtypes = [i64, i64, i32, c.c_int, vp]
    L.actq_sample_sensitivity.restype = c.c_int
    L.actq_sample_sensitivity.argtypes = [vp, i64, i64, i32, vp, vp, vp]
    L.actq_allocate_bits.restype = c.c_int
    L.actq_allocate_bits.argtypes = [vp, vp, i64, i64, c.c_uint32, vp]
    L.actq_group_stats_multi.restype = c.c_int
    L.actq_group_stats_multi.argtypes = [vp, i32, c.c_int, i64, i32, vp]
    L.actq_quantize_pack_multi.restype = c.c_int
    L.actq_quantize_pack_multi.argtypes = [vp, i32, c.c_int, i64, i32, u64, u64, i32, vp, u64, c.c_int, vp]
    L.actq_unpack_dequantize_multi.restype = c.c_int
    L.actq_unpack_dequantize_multi.argtypes = [vp, i32, vp, u64, c.c_int, i64, i32, c.c_int, vp]
    L.actq_tensor_stats.restype = c.c_int
    L.actq_tensor_stats.argtypes = [vp, c.c_int, i64, vp, vp]
    L.actq_relu_mask_bytes.restype = c.c_int
    L.actq_relu_mask_bytes.argtypes = [i64, vp]
    L.actq_relu_forward.restype = c.c_int
    L.actq_relu_forward.argtypes = [vp, c.c_int, i64, vp, vp, vp]
    L.actq_relu_backward.restype = c.c_int
    L.actq_relu_backward.argtypes = [vp, vp, c.c_int, i64, vp, vp]
    L.actq_pool2d_output_size.restype = c.c_int
    L.actq_pool2d_output_size.argtypes = [i32] * 10 + [vp, vp]
    L.actq_maxpool2d_forward.restype = c.c_int
    L.actq_maxpool2d_forward.argtypes = [vp, c.c_int, i64] + [i32] * 10 + [vp, vp, vp]
    L.actq_maxpool2d_backward.restype = c.c_int
    L.actq_maxpool2d_backward.argtypes = [vp, vp, c.c_int, i64] + [i32] * 10 + [vp, vp]
    L.actq_allocate_bits_device.restype = c.c_int
    L.actq_allocate_bits_device.argtypes = [vp, vp, i64, i64, i32, i64, c.c_uint32, vp, vp, vp, vp]
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != ACTQ_OK:
        raise ActqError(rc, lib().actq_last_error().decode())


def _torch():
    import torch
    return torch


def _dtype_code(t) -> int:
    torch = _torch()
    if t.dtype == torch.float32:
        return ACTQ_F32
    if t.dtype == torch.float16:
        return ACTQ_F16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t, dtype=None, name="tensor"):
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream(stream) -> int:
    torch = _torch()
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _view2d(x):
    return int(x.shape[0]), int(x.numel() // x.shape[0])


def version() -> int:
    return lib().actq_version()


def last_error() -> str:
    return lib().actq_last_error().decode()


def packed_bytes(N: int, D: int, bits_host, G: int = G_DEFAULT):
    """Host: (offsets uint64[N], total bytes) of the bit stream for widths bits_host."""
    bits = np.ascontiguousarray(bits_host, dtype=np.uint8)
    if bits.shape != (N,):
        raise ValueError("bits must have shape [N]")
    offsets = np.zeros(N, dtype=np.uint64)
    total = ctypes.c_uint64(0)
    _check(lib().actq_packed_bytes(N, D, G, bits.ctypes.data, offsets.ctypes.data, ctypes.addressof(total)))
    return offsets, int(total.value)


def group_stats(x, gmin=None, grange=None, G: int = G_DEFAULT, stream=None):
    """Device: per-group (min, range) of x viewed as [N, D]; returns float32 [N, ng] tensors."""
    torch = _torch()
    N, D = _view2d(x)
    ng = (D + G - 1) // G
    if gmin is None:
        gmin = torch.empty((N, ng), dtype=torch.float32, device=x.device)
    if grange is None:
        grange = torch.empty((N, ng), dtype=torch.float32, device=x.device)
    if gmin.numel() != N * ng or grange.numel() != N * ng:
        raise ValueError("gmin / grange must hold N*ng floats")
    _check(lib().actq_group_stats(_dev(x, name="x"), _dtype_code(x), N, D, G,
                                  _dev(gmin, torch.float32, "gmin"), _dev(grange, torch.float32, "grange"),
                                  _stream(stream)))
    return gmin, grange


def header_bytes(N: int, D: int, hf: int = ACTQ_HDR_F32, G: int = G_DEFAULT) -> int:
    out = ctypes.c_uint64(0)
    _check(lib().actq_header_bytes(N, D, G, hf, ctypes.addressof(out)))
    return int(out.value)


def _header_ptr(header, N, ng, hf):
    torch = _torch()
    want = torch.int16 if hf == ACTQ_HDR_BF16 else torch.float32
    if header.dtype != want:
        raise TypeError(f"header must be {want} for this header format, got {header.dtype}")
    if header.numel() != (2 if hf == ACTQ_HDR_TENSOR else N * ng * 2):
        raise ValueError("header must hold N*ng*2 entries (2 for ACTQ_HDR_TENSOR)")
    return _dev(header, want, "header")


def quantize_pack(x, bits, offsets, packed, header, seed: int, tag: int = 0, noise_bits: int = 24,
                  G: int = G_DEFAULT, stream=None, hf: int = ACTQ_HDR_F32):
    """Device: writes the bit stream into `packed` (uint8) and the group headers into `header`
    (float32 [N*ng*2] for ACTQ_HDR_F32, int16 [N*ng*2] bfloat16 bit patterns for ACTQ_HDR_BF16).
    With ACTQ_HDR_TENSOR `header` is the float32 [2] pair from tensor_stats and is only read."""
    torch = _torch()
    N, D = _view2d(x)
    ng = (D + G - 1) // G
    if bits.numel() != N or offsets.numel() != N:
        raise ValueError("bits and offsets must have N entries")
    _check(lib().actq_quantize_pack(_dev(x, name="x"), _dtype_code(x), N, D, G,
                                    _dev(bits, torch.uint8, "bits"), _dev(offsets, torch.int64, "offsets"),
                                    seed & (2 ** 64 - 1), tag & (2 ** 64 - 1), noise_bits,
                                    _dev(packed, torch.uint8, "packed"), packed.numel(),
                                    _header_ptr(header, N, ng, hf), hf, _stream(stream)))
    return packed, header


def unpack_dequantize(packed, header, bits, offsets, out, G: int = G_DEFAULT, stream=None,
                      hf: int = ACTQ_HDR_F32):
    """Device: reconstructs `out` ([N, ...] float32 or float16) from the bit stream."""
    torch = _torch()
    N, D = _view2d(out)
    ng = (D + G - 1) // G
    if bits.numel() != N or offsets.numel() != N:
        raise ValueError("bits and offsets must have N entries")
    _check(lib().actq_unpack_dequantize(_dev(packed, torch.uint8, "packed"), packed.numel(),
                                        _header_ptr(header, N, ng, hf), hf,
                                        _dev(bits, torch.uint8, "bits"), _dev(offsets, torch.int64, "offsets"),
                                        N, D, G, _dev(out, name="out"), _dtype_code(out), _stream(stream)))
    return out


def sample_sensitivity(grange, grad2=None, w=None, G: int = G_DEFAULT, stream=None):
    """Device: w[n] = (G/6) * grad2[n] * sum_g grange[n, g]^2 (grad2 = None means 1)."""
    torch = _torch()
    if grange.dim() != 2:
        raise ValueError("grange must be [N, ng]")
    N, ng = int(grange.shape[0]), int(grange.shape[1])
    if w is None:
        w = torch.empty(N, dtype=torch.float32, device=grange.device)
    if w.numel() != N or (grad2 is not None and grad2.numel() != N):
        raise ValueError("w and grad2 must have N entries")
    g2 = None if grad2 is None else _dev(grad2, torch.float32, "grad2")
    _check(lib().actq_sample_sensitivity(_dev(grange, torch.float32, "grange"), N, ng, G, g2,
                                         _dev(w, torch.float32, "w"), _stream(stream)))
    return w


def allocate_bits(w_host, D_host, budget_bits: int, widths: int = ACTQ_WIDTHS_POW2) -> np.ndarray:
    """Host: greedy widths (from the set `widths`, bit b = b bits) for sensitivities w and sizes D
    under a bit budget."""
    w = np.ascontiguousarray(w_host, dtype=np.float32)
    D = np.ascontiguousarray(D_host, dtype=np.int64)
    if w.ndim != 1 or D.shape != w.shape:
        raise ValueError("w and D must be 1-D arrays of equal length")
    bits = np.zeros(w.shape[0], dtype=np.uint8)
    rc = lib().actq_allocate_bits(w.ctypes.data, D.ctypes.data, w.shape[0], int(budget_bits), int(widths),
                                  bits.ctypes.data)
    if rc != ACTQ_OK:
        err = ActqError(rc, lib().actq_last_error().decode())
        err.bits = bits
        raise err
    return bits


def allocate_bits_device(w, D, budget_bits: int, widths: int = ACTQ_WIDTHS_POW2, bits=None, offsets=None,
                         result=None, G: int = G_DEFAULT, stream=None):
    """Device: the same greedy allocation without a host round trip.  `w` is a float32 device
    tensor [M]; `D` is an int (every item has D elements) or an int64 device tensor [M].
    Returns (bits uint8 [M], offsets int64 [M], result int64 [2] = total bytes, status); nothing
    is synchronised, so the status is the caller's to read when convenient."""
    torch = _torch()
    M = int(w.numel())
    if bits is None:
        bits = torch.empty(M, dtype=torch.uint8, device=w.device)
    if offsets is None:
        offsets = torch.empty(M, dtype=torch.int64, device=w.device)
    if result is None:
        result = torch.empty(2, dtype=torch.int64, device=w.device)
    if bits.numel() != M or offsets.numel() != M or result.numel() != 2:
        raise ValueError("bits and offsets must have M entries, result 2")
    if isinstance(D, int):
        d_items, d_uniform = None, D
    else:
        if D.numel() != M:
            raise ValueError("D must have M entries")
        d_items, d_uniform = _dev(D, torch.int64, "D"), 0
    _check(lib().actq_allocate_bits_device(_dev(w, torch.float32, "w"), d_items, d_uniform, M, G,
                                           int(budget_bits), int(widths), _dev(bits, torch.uint8, "bits"),
                                           _dev(offsets, torch.int64, "offsets"),
                                           _dev(result, torch.int64, "result"), _stream(stream)))
    return bits, offsets, result


# ----------------------------------------------------------------------------- exact layer contexts

def relu_mask_bytes(n: int) -> int:
    out = ctypes.c_uint64()
    _check(lib().actq_relu_mask_bytes(int(n), ctypes.addressof(out)))
    return out.value


def relu_forward(x, y=None, mask=None, stream=None):
    """Device: y = max(x, 0) and the 1-bit context.  Returns (y, mask uint8)."""
    torch = _torch()
    n = int(x.numel())
    if y is None:
        y = torch.empty_like(x)
    if mask is None:
        mask = torch.empty(relu_mask_bytes(n), dtype=torch.uint8, device=x.device)
    if y.numel() != n or y.dtype != x.dtype or mask.numel() != relu_mask_bytes(n):
        raise ValueError("y must match x and mask must have relu_mask_bytes(n) bytes")
    _check(lib().actq_relu_forward(_dev(x, None, "x"), _dtype_code(x), n, _dev(y, None, "y"),
                                   _dev(mask, torch.uint8, "mask"), _stream(stream)))
    return y, mask


def relu_backward(mask, grad_y, grad_x=None, stream=None):
    """Device: grad_x = grad_y where the stored bit is set, +0 elsewhere."""
    torch = _torch()
    n = int(grad_y.numel())
    if grad_x is None:
        grad_x = torch.empty_like(grad_y)
    if grad_x.numel() != n or grad_x.dtype != grad_y.dtype or mask.numel() != relu_mask_bytes(n):
        raise ValueError("grad_x must match grad_y and mask must have relu_mask_bytes(n) bytes")
    _check(lib().actq_relu_backward(_dev(mask, torch.uint8, "mask"), _dev(grad_y, None, "grad_y"), _dtype_code(grad_y),
                                    n, _dev(grad_x, None, "grad_x"), _stream(stream)))
    return grad_x


def pool2d_output_size(H, W, kernel, stride, padding=(0, 0), dilation=(1, 1)):
    oh, ow = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().actq_pool2d_output_size(H, W, *kernel, *stride, *padding, *dilation,
                                         ctypes.addressof(oh), ctypes.addressof(ow)))
    return oh.value, ow.value


def maxpool2d_forward(x, kernel, stride, padding=(0, 0), dilation=(1, 1), y=None, argmax=None, stream=None):
    """Device: x [..., H, W] -> (y [..., OH, OW], argmax uint8 [..., OH, OW])."""
    torch = _torch()
    H, W = int(x.shape[-2]), int(x.shape[-1])
    planes = int(x.numel() // (H * W))
    OH, OW = pool2d_output_size(H, W, kernel, stride, padding, dilation)
    shape = tuple(x.shape[:-2]) + (OH, OW)
    if y is None:
        y = torch.empty(shape, dtype=x.dtype, device=x.device)
    if argmax is None:
        argmax = torch.empty(shape, dtype=torch.uint8, device=x.device)
    if y.numel() != planes * OH * OW or argmax.numel() != planes * OH * OW or y.dtype != x.dtype:
        raise ValueError("y and argmax must have planes*OH*OW elements")
    _check(lib().actq_maxpool2d_forward(_dev(x, None, "x"), _dtype_code(x), planes, H, W, *kernel, *stride, *padding,
                                        *dilation, _dev(y, None, "y"), _dev(argmax, torch.uint8, "argmax"),
                                        _stream(stream)))
    return y, argmax


def maxpool2d_backward(argmax, grad_y, H, W, kernel, stride, padding=(0, 0), dilation=(1, 1), grad_x=None,
                       stream=None):
    """Device: gradient of the input from the stored window positions."""
    torch = _torch()
    OH, OW = pool2d_output_size(H, W, kernel, stride, padding, dilation)
    if tuple(grad_y.shape[-2:]) != (OH, OW) or argmax.numel() != grad_y.numel():
        raise ValueError("grad_y and argmax must be [..., OH, OW]")
    planes = int(grad_y.numel() // (OH * OW))
    if grad_x is None:
        grad_x = torch.empty(tuple(grad_y.shape[:-2]) + (H, W), dtype=grad_y.dtype, device=grad_y.device)
    if grad_x.numel() != planes * H * W or grad_x.dtype != grad_y.dtype:
        raise ValueError("grad_x must have planes*H*W elements")
    _check(lib().actq_maxpool2d_backward(_dev(argmax, torch.uint8, "argmax"), _dev(grad_y, None, "grad_y"),
                                         _dtype_code(grad_y), planes, H, W, *kernel, *stride, *padding, *dilation,
                                         _dev(grad_x, None, "grad_x"), _stream(stream)))
    return grad_x


def tensor_stats(x, zr=None, stream=None):
    """Device: (Z, R) = (min, max - min) of the whole tensor, float32 [2]: the header of ACTQ_HDR_TENSOR."""
    torch = _torch()
    if zr is None:
        zr = torch.empty(2, dtype=torch.float32, device=x.device)
    if zr.numel() != 2:
        raise ValueError("zr must have two entries")
    _check(lib().actq_tensor_stats(_dev(x, None, "x"), _dtype_code(x), int(x.numel()), _dev(zr, torch.float32, "zr"),
                                   _stream(stream)))
    return zr


# ----------------------------------------------------------------------------- several tensors per launch

MAX_TENSORS_PER_CALL = 40


class TensorDesc(ctypes.Structure):
    """Mirror of `actq_tensor` (include/actq.h)."""
    _fields_ = [("x", ctypes.c_void_p), ("out", ctypes.c_void_p), ("gmin", ctypes.c_void_p),
                ("grange", ctypes.c_void_p), ("header", ctypes.c_void_p), ("bits", ctypes.c_void_p),
                ("offsets", ctypes.c_void_p), ("D", ctypes.c_int64)]


def tensor_table(entries):
    """Host-side descriptor array from dicts with any of the keys x, out, gmin, grange, header, bits,
    offsets (device tensors) and D.  All tensors must be [N, D] views with the same N."""
    torch = _torch()
    table = (TensorDesc * len(entries))()
    for slot, e in zip(table, entries):
        for key in ("x", "out", "gmin", "grange", "header", "bits", "offsets"):
            t = e.get(key)
            setattr(slot, key, None if t is None else _dev(t, None, key))
        slot.D = int(e["D"])
    return table


def group_stats_multi(table, dtype_code: int, N: int, G: int = G_DEFAULT, stream=None):
    _check(lib().actq_group_stats_multi(ctypes.addressof(table), len(table), dtype_code, N, G, _stream(stream)))


def quantize_pack_multi(table, dtype_code: int, N: int, packed, seed: int, tag: int = 0, noise_bits: int = 24,
                        G: int = G_DEFAULT, stream=None, hf: int = ACTQ_HDR_F32):
    torch = _torch()
    _check(lib().actq_quantize_pack_multi(ctypes.addressof(table), len(table), dtype_code, N, G, seed, tag, noise_bits,
                                          _dev(packed, torch.uint8, "packed"), int(packed.numel()), hf,
                                          _stream(stream)))


def unpack_dequantize_multi(table, dtype_code: int, N: int, packed, G: int = G_DEFAULT, stream=None,
                            hf: int = ACTQ_HDR_F32):
    torch = _torch()
    _check(lib().actq_unpack_dequantize_multi(ctypes.addressof(table), len(table), _dev(packed, torch.uint8, "packed"),
                                              int(packed.numel()), hf, N, G, dtype_code, _stream(stream)))
