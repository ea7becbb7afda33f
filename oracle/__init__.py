"""CPU oracle for the ActNN activation-compression hot path -- TEST INFRASTRUCTURE.

This package compiles ``actq_oracle.c`` with gcc and exposes it on numpy arrays.
It is independent of the GPU library: it imports nothing from
``paper_2104_14129_amd`` and that package imports nothing from here.  Only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may use it.

Passages followed: Sec. 4.1 (per-group quantization, stochastic rounding,
dequantization), Sec. 4.2 Prob. (9) and Sec. 4.3 (greedy bit allocation).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "actq_oracle.c")
_LIB = os.path.join(_HERE, "libactq_oracle.so")

F32, F16 = 0, 1
OK, EINVAL, EINFEASIBLE = 0, -1, -2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no contraction of a*b+c, OpenMP over groups)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".{os.getpid()}.tmp"
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared",
               "-fPIC", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        c = ctypes
        vp, i64, i32, u64 = c.c_void_p, c.c_int64, c.c_int32, c.c_uint64
        L.orc_half_to_float.restype = c.c_float
        L.orc_half_to_float.argtypes = [c.c_uint16]
        L.orc_float_to_half.restype = c.c_uint16
        L.orc_float_to_half.argtypes = [c.c_float]
        L.orc_philox4x32_10.restype = None
        L.orc_philox4x32_10.argtypes = [vp, vp, vp]
        L.orc_noise.restype = c.c_float
        L.orc_noise.argtypes = [u64, u64, c.c_uint32, u64, c.c_int]
        L.orc_packed_bytes.restype = c.c_int
        L.orc_packed_bytes.argtypes = [i64, i64, i32, vp, vp, vp]
        L.orc_group_stats.restype = c.c_int
        L.orc_group_stats.argtypes = [vp, c.c_int, i64, i64, i32, vp, vp]
        L.orc_quantize_pack.restype = c.c_int
        L.orc_quantize_pack.argtypes = [vp, c.c_int, i64, i64, i32, vp, vp, u64, u64, i32, vp, vp]
        L.orc_quantize_group.restype = c.c_int
        L.orc_quantize_group.argtypes = [vp, c.c_int, i64, i64, i32, c.c_int, u64, u64, c.c_uint32, u64, i32, vp, vp]
        L.orc_dequantize_group.restype = c.c_int
        L.orc_dequantize_group.argtypes = [vp, vp, c.c_int, i64, vp, c.c_int, i64]
        L.orc_bf16_to_float.restype = c.c_float
        L.orc_bf16_to_float.argtypes = [c.c_uint16]
        L.orc_bf16_floor.restype = c.c_uint16
        L.orc_bf16_floor.argtypes = [c.c_float]
        L.orc_bf16_ceil.restype = c.c_uint16
        L.orc_bf16_ceil.argtypes = [c.c_float]
        L.orc_quantize_pack_bf16.restype = c.c_int
        L.orc_quantize_pack_bf16.argtypes = [vp, c.c_int, i64, i64, i32, vp, vp, u64, u64, i32, vp, vp]
        L.orc_unpack_dequantize_bf16.restype = c.c_int
        L.orc_unpack_dequantize_bf16.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, c.c_int]
        L.orc_sample_sensitivity.restype = c.c_int
        L.orc_sample_sensitivity.argtypes = [vp, i64, i64, i32, vp, vp]
        L.orc_quantize_codes.restype = c.c_int
        L.orc_quantize_codes.argtypes = [vp, c.c_int, i64, i64, i32, vp, u64, u64, i32, vp]
        L.orc_unpack_dequantize.restype = c.c_int
        L.orc_unpack_dequantize.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, c.c_int]
        L.orc_allocate_bits.restype = c.c_int
        L.orc_allocate_bits.argtypes = [vp, vp, i64, i64, vp]
        L.orc_allocate_bits_ladder.restype = c.c_int
        L.orc_allocate_bits_ladder.argtypes = [vp, vp, i64, i64, c.c_uint32, vp]
        i32 = c.c_int32
        L.orc_relu_forward.restype = c.c_int
        L.orc_relu_forward.argtypes = [vp, c.c_int, i64, vp, vp]
        L.orc_relu_backward.restype = c.c_int
        L.orc_relu_backward.argtypes = [vp, vp, c.c_int, i64, vp]
        L.orc_pool2d_output_size.restype = c.c_int
        L.orc_pool2d_output_size.argtypes = [i32] * 10 + [vp, vp]
        L.orc_maxpool2d_forward.restype = c.c_int
        L.orc_maxpool2d_forward.argtypes = [vp, c.c_int, i64] + [i32] * 10 + [vp, vp]
        L.orc_maxpool2d_backward.restype = c.c_int
        L.orc_maxpool2d_backward.argtypes = [vp, vp, c.c_int, i64] + [i32] * 10 + [vp]
        L.orc_tensor_stats.restype = c.c_int
        L.orc_tensor_stats.argtypes = [vp, c.c_int, i64, vp]
        L.orc_quantize_pack_tensor.restype = c.c_int
        L.orc_quantize_pack_tensor.argtypes = [vp, c.c_int, i64, i64, c.c_int32, vp, vp, u64, u64, c.c_int32, vp, vp]
        L.orc_unpack_dequantize_tensor.restype = c.c_int
        L.orc_unpack_dequantize_tensor.argtypes = [vp, vp, vp, vp, i64, i64, c.c_int32, vp, c.c_int]
        L.orc_objective.restype = c.c_double
        L.orc_objective.argtypes = [vp, vp, i64]
        _lib = L
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"oracle {what} failed with code {code}")
        self.code = code


def _p(a: np.ndarray) -> int:
    return a.ctypes.data


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"unsupported dtype {a.dtype}")


def _as2d(x: np.ndarray):
    x = np.ascontiguousarray(x)
    n = x.shape[0]
    return x.reshape(n, -1)


def threads() -> int:
    """Number of OpenMP threads the oracle's loops will use."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return os.cpu_count() or 1


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def noise(seed: int, tag: int, n: int, d: int, noise_bits: int = 24) -> float:
    return float(lib().orc_noise(seed, tag, n, d, noise_bits))


def half_to_float(h: int) -> float:
    return float(lib().orc_half_to_float(h))


def float_to_half(f: float) -> int:
    return int(lib().orc_float_to_half(f))


def packed_bytes(N: int, D: int, G: int, bits) -> tuple[np.ndarray, int]:
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    offsets = np.zeros(max(N, 1), dtype=np.uint64)
    total = ctypes.c_uint64(0)
    rc = lib().orc_packed_bytes(N, D, G, _p(bits), _p(offsets), ctypes.addressof(total))
    if rc != OK:
        raise OracleError(rc, "packed_bytes")
    return offsets[:N], int(total.value)


def group_stats(x: np.ndarray, G: int = 256) -> tuple[np.ndarray, np.ndarray]:
    """Per-group (min, range) of an [N, ...] tensor, each [N, ng] float32."""
    x2 = _as2d(x)
    N, D = x2.shape
    ng = (D + G - 1) // G
    gmin = np.empty((N, ng), dtype=np.float32)
    grange = np.empty((N, ng), dtype=np.float32)
    rc = lib().orc_group_stats(_p(x2), _dtype_code(x2), N, D, G, _p(gmin), _p(grange))
    if rc != OK:
        raise OracleError(rc, "group_stats")
    return gmin, grange


def quantize_pack(x: np.ndarray, bits, seed: int, tag: int = 0, G: int = 256,
                  noise_bits: int = 24):
    """Returns (packed uint8[total], header float32[N, ng, 2], offsets uint64[N])."""
    x2 = _as2d(x)
    N, D = x2.shape
    ng = (D + G - 1) // G
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    offsets, total = packed_bytes(N, D, G, bits)
    packed = np.full(total, 0xFF, dtype=np.uint8)   # every byte of the stream must come from the oracle
    header = np.empty((N, ng, 2), dtype=np.float32)
    rc = lib().orc_quantize_pack(_p(x2), _dtype_code(x2), N, D, G, _p(bits), _p(offsets),
                                 seed, tag, noise_bits, _p(packed), _p(header))
    if rc != OK:
        raise OracleError(rc, "quantize_pack")
    return packed, header, offsets


HDR_F32, HDR_BF16 = 0, 1


def bf16_floor(f: float) -> int:
    return int(lib().orc_bf16_floor(f))


def bf16_ceil(f: float) -> int:
    return int(lib().orc_bf16_ceil(f))


def bf16_to_float(h: int) -> float:
    return float(lib().orc_bf16_to_float(h))


def quantize_pack_bf16(x: np.ndarray, bits, seed: int, tag: int = 0, G: int = 256, noise_bits: int = 24):
    """As quantize_pack, with the header stored as bfloat16 (Z rounded down, R rounded up):
    returns (packed uint8[total], header uint16[N, ng, 2] = (Z, R) bit patterns, offsets)."""
    x2 = _as2d(x)
    N, D = x2.shape
    ng = (D + G - 1) // G
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    offsets, total = packed_bytes(N, D, G, bits)
    packed = np.full(total, 0xFF, dtype=np.uint8)   # every byte of the stream must come from the oracle
    header = np.empty((N, ng, 2), dtype=np.uint16)
    rc = lib().orc_quantize_pack_bf16(_p(x2), _dtype_code(x2), N, D, G, _p(bits), _p(offsets),
                                      seed, tag, noise_bits, _p(packed), _p(header))
    if rc != OK:
        raise OracleError(rc, "quantize_pack_bf16")
    return packed, header, offsets


def unpack_dequantize_bf16(packed, header, bits, offsets, N: int, D: int, G: int = 256, out_dtype=np.float32):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    header = np.ascontiguousarray(header, dtype=np.uint16)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    out = np.empty((N, D), dtype=out_dtype)
    rc = lib().orc_unpack_dequantize_bf16(_p(packed), _p(header), _p(bits), _p(offsets), N, D, G,
                                          _p(out), _dtype_code(out))
    if rc != OK:
        raise OracleError(rc, "unpack_dequantize_bf16")
    return out


def sample_sensitivity(grange: np.ndarray, G: int = 256, grad2=None) -> np.ndarray:
    """w_n = (G/6) * grad2_n * sum_g R_ng^2 (grad2 = None means 1), float32 [N]."""
    grange = np.ascontiguousarray(grange, dtype=np.float32)
    N, ng = grange.shape
    w = np.empty(N, dtype=np.float32)
    g2 = None if grad2 is None else np.ascontiguousarray(grad2, dtype=np.float32)
    rc = lib().orc_sample_sensitivity(_p(grange), N, ng, G, None if g2 is None else _p(g2), _p(w))
    if rc != OK:
        raise OracleError(rc, "sample_sensitivity")
    return w


def quantize_group(xg: np.ndarray, b: int, seed: int, tag: int, n: int, d_start: int,
                   G: int = 256, noise_bits: int = 24):
    """One group (len(xg) <= G valid elements of sample n starting at feature d_start):
    returns (bytes uint8[G*b/8], header float32[2])."""
    xg = np.ascontiguousarray(xg).reshape(-1)
    dst = np.zeros(G * b // 8, dtype=np.uint8)
    hd = np.zeros(2, dtype=np.float32)
    rc = lib().orc_quantize_group(_p(xg), _dtype_code(xg), 0, xg.size, G, b, seed, tag, n, d_start,
                                  noise_bits, _p(dst), _p(hd))
    if rc != OK:
        raise OracleError(rc, "quantize_group")
    return dst, hd


def dequantize_group(src: np.ndarray, hd: np.ndarray, b: int, length: int, out_dtype=np.float32) -> np.ndarray:
    src = np.ascontiguousarray(src, dtype=np.uint8)
    hd = np.ascontiguousarray(hd, dtype=np.float32)
    out = np.empty(length, dtype=out_dtype)
    rc = lib().orc_dequantize_group(_p(src), _p(hd), b, length, _p(out), _dtype_code(out), 0)
    if rc != OK:
        raise OracleError(rc, "dequantize_group")
    return out


def quantize_codes(x: np.ndarray, bits, seed: int, tag: int = 0, G: int = 256,
                   noise_bits: int = 24) -> np.ndarray:
    """The integer codes themselves, uint8[N, D] (no packing)."""
    x2 = _as2d(x)
    N, D = x2.shape
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    codes = np.empty((N, D), dtype=np.uint8)
    rc = lib().orc_quantize_codes(_p(x2), _dtype_code(x2), N, D, G, _p(bits), seed, tag,
                                  noise_bits, _p(codes))
    if rc != OK:
        raise OracleError(rc, "quantize_codes")
    return codes


def unpack_dequantize(packed: np.ndarray, header: np.ndarray, bits, offsets,
                      N: int, D: int, G: int = 256, out_dtype=np.float32) -> np.ndarray:
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    header = np.ascontiguousarray(header, dtype=np.float32)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    out = np.empty((N, D), dtype=out_dtype)
    rc = lib().orc_unpack_dequantize(_p(packed), _p(header), _p(bits), _p(offsets), N, D, G,
                                     _p(out), _dtype_code(out))
    if rc != OK:
        raise OracleError(rc, "unpack_dequantize")
    return out


WIDTHS_POW2 = 0x116  # {1, 2, 4, 8}
WIDTHS_ALL = 0x1FE   # {1, ..., 8}


def allocate_bits(w, D, budget_bits: int, widths: int = WIDTHS_POW2) -> np.ndarray:
    """Greedy allocation over the widths whose bit is set in `widths` (bit b: b bits)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    D = np.ascontiguousarray(D, dtype=np.int64)
    bits = np.zeros(w.shape[0], dtype=np.uint8)
    rc = lib().orc_allocate_bits_ladder(_p(w), _p(D), w.shape[0], int(budget_bits), int(widths), _p(bits))
    if rc != OK:
        err = OracleError(rc, "allocate_bits")
        err.bits = bits
        raise err
    return bits


def objective(w, bits) -> float:
    w = np.ascontiguousarray(w, dtype=np.float32)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    return float(lib().orc_objective(_p(w), _p(bits), w.shape[0]))


# ----------------------------------------------------------------------------- exact contexts

def relu_forward(x: np.ndarray):
    """y = x where x > 0 else +0, and the 1-bit context (uint8, ceil(n/256)*32 bytes)."""
    x = np.ascontiguousarray(x)
    y = np.empty_like(x)
    mask = np.empty((x.size + 255) // 256 * 32, dtype=np.uint8)
    rc = lib().orc_relu_forward(_p(x), _dtype_code(x), x.size, _p(y), _p(mask))
    if rc != OK:
        raise OracleError(rc, "relu_forward")
    return y, mask


def relu_backward(mask: np.ndarray, grad_y: np.ndarray) -> np.ndarray:
    grad_y = np.ascontiguousarray(grad_y)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    gx = np.empty_like(grad_y)
    rc = lib().orc_relu_backward(_p(mask), _p(grad_y), _dtype_code(grad_y), grad_y.size, _p(gx))
    if rc != OK:
        raise OracleError(rc, "relu_backward")
    return gx


def pool2d_output_size(H, W, kernel, stride, padding=(0, 0), dilation=(1, 1)):
    import ctypes as c
    oh, ow = c.c_int32(), c.c_int32()
    rc = lib().orc_pool2d_output_size(H, W, *kernel, *stride, *padding, *dilation, c.addressof(oh), c.addressof(ow))
    if rc != OK:
        raise OracleError(rc, "pool2d_output_size")
    return oh.value, ow.value


def maxpool2d_forward(x: np.ndarray, kernel, stride, padding=(0, 0), dilation=(1, 1)):
    """x [..., H, W] -> (y [..., OH, OW], argmax uint8 [..., OH, OW] = position inside the window)."""
    x = np.ascontiguousarray(x)
    H, W = x.shape[-2:]
    planes = x.size // (H * W)
    OH, OW = pool2d_output_size(H, W, kernel, stride, padding, dilation)
    y = np.empty(x.shape[:-2] + (OH, OW), dtype=x.dtype)
    arg = np.empty(y.shape, dtype=np.uint8)
    rc = lib().orc_maxpool2d_forward(_p(x), _dtype_code(x), planes, H, W, *kernel, *stride, *padding, *dilation,
                                     _p(y), _p(arg))
    if rc != OK:
        raise OracleError(rc, "maxpool2d_forward")
    return y, arg


def maxpool2d_backward(argmax: np.ndarray, grad_y: np.ndarray, H: int, W: int, kernel, stride,
                       padding=(0, 0), dilation=(1, 1)) -> np.ndarray:
    grad_y = np.ascontiguousarray(grad_y)
    argmax = np.ascontiguousarray(argmax, dtype=np.uint8)
    OH, OW = grad_y.shape[-2:]
    planes = grad_y.size // (OH * OW)
    gx = np.empty(grad_y.shape[:-2] + (H, W), dtype=grad_y.dtype)
    rc = lib().orc_maxpool2d_backward(_p(argmax), _p(grad_y), _dtype_code(grad_y), planes, H, W, *kernel, *stride,
                                      *padding, *dilation, _p(gx))
    if rc != OK:
        raise OracleError(rc, "maxpool2d_backward")
    return gx


# ----------------------------------------------------------------------------- per-tensor baseline

def tensor_stats(x: np.ndarray) -> np.ndarray:
    """float32 [2]: (Z, R) = (min, max - min) over the whole tensor."""
    x = np.ascontiguousarray(x)
    zr = np.empty(2, dtype=np.float32)
    rc = lib().orc_tensor_stats(_p(x), _dtype_code(x), x.size, _p(zr))
    if rc != OK:
        raise OracleError(rc, "tensor_stats")
    return zr


def quantize_pack_tensor(x: np.ndarray, bits, zr, seed: int, tag: int = 0, G: int = 256, noise_bits: int = 24):
    """Per-tensor quantizer: one (Z, R) for all groups.  Returns (packed, offsets)."""
    x = _as2d(x)
    N, D = x.shape
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    zr = np.ascontiguousarray(zr, dtype=np.float32)
    offsets, total = packed_bytes(N, D, G, bits)
    packed = np.full(total, 0xFF, dtype=np.uint8)   # every byte of the stream must come from the oracle
    rc = lib().orc_quantize_pack_tensor(_p(x), _dtype_code(x), N, D, G, _p(bits), _p(offsets), seed, tag,
                                        noise_bits, _p(zr), _p(packed))
    if rc != OK:
        raise OracleError(rc, "quantize_pack_tensor")
    return packed, offsets


def unpack_dequantize_tensor(packed, zr, bits, offsets, N: int, D: int, G: int = 256, out_dtype=np.float32):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    zr = np.ascontiguousarray(zr, dtype=np.float32)
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    offsets = np.ascontiguousarray(offsets, dtype=np.uint64)
    out = np.empty((N, D), dtype=out_dtype)
    rc = lib().orc_unpack_dequantize_tensor(_p(packed), _p(zr), _p(bits), _p(offsets), N, D, G, _p(out),
                                            _dtype_code(out))
    if rc != OK:
        raise OracleError(rc, "unpack_dequantize_tensor")
    return out
