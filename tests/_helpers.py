"""Small test-side utilities (no method arithmetic shared with the oracle or the kernels)."""
from __future__ import annotations

import os
import shutil
import subprocess
from fractions import Fraction

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def round_fraction_to_f32(fr: Fraction) -> np.float32:
    """Correctly rounded (nearest, ties to even) binary32 value of an exact rational."""
    if fr == 0:
        return np.float32(0.0)
    cand = np.float32(float(fr))          # may be off by one ulp (double rounding)
    best = None
    for c in (np.nextafter(cand, np.float32(-np.inf)), cand, np.nextafter(cand, np.float32(np.inf))):
        if not np.isfinite(c):
            continue
        err = abs(Fraction(float(c)) - fr)
        even = (int(np.float32(c).view(np.uint32)) & 1) == 0
        key = (err, 0 if even else 1)
        if best is None or key < best[0]:
            best = (key, c)
    return np.float32(best[1])


_WITNESS = None


def philox_witness():
    """Path of the compiled rocRAND host witness, or None when hipcc / rocRAND are absent."""
    global _WITNESS
    if _WITNESS is not None:
        return _WITNESS or None
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    src = os.path.join(ROOT, "tests", "witness", "rocrand_philox_witness.cpp")
    out = os.path.join(ROOT, "tests", "witness", "rocrand_philox_witness.bin")
    if not os.path.exists(hipcc) or not os.path.exists("/opt/rocm/include/rocrand/rocrand_philox4x32_10.h"):
        _WITNESS = ""
        return None
    if not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        r = subprocess.run([hipcc, "--offload-host-only", "-O1", "-o", out, src],
                           capture_output=True, text=True)
        if r.returncode != 0:
            _WITNESS = ""
            return None
    _WITNESS = out
    return out


def witness_words(queries):
    """queries: list of (seed, subsequence, offset) -> uint32 array [len, 4] from rocRAND."""
    exe = philox_witness()
    assert exe is not None
    text = "".join(f"{s:#x} {sub:#x} {off:#x}\n" for s, sub, off in queries)
    r = subprocess.run([exe], input=text, capture_output=True, text=True, check=True)
    rows = [[int(t, 16) for t in line.split()] for line in r.stdout.strip().splitlines()]
    return np.array(rows, dtype=np.uint32).reshape(len(queries), 4)


def witness_noise_words(seed: int, tag: int, n: int, counter0: int) -> np.ndarray:
    """The four Philox words at counter (counter0, n, lo32(tag), hi32(tag)), key = seed.

    rocRAND's state is a 128-bit counter whose low 64 bits advance by offset/4 and whose
    high 64 bits hold the subsequence, and its key is the seed: so subsequence = tag and
    offset = 4 * (counter0 + n * 2^32).
    """
    off = 4 * (counter0 + (n << 32))
    assert off < (1 << 64)
    return witness_words([(seed, tag, off)])[0]


def clamp_case(noise_bits: int, seed: int = 321, D: int = 1 << 18):
    """A one-sample tensor of D elements (8 bits) whose group maxima overshoot B = 255 by one
    ulp after the two roundings of (h - Z) * (B / R), placed on exactly those elements whose
    noise is extreme enough to turn the overshoot into code 256 if the scaled value were not
    clamped (Sec. 4.1 scaling; noise below that ulp when compared, within that ulp of 1 when
    added).  Returns (x [1, D] float32, the indices of those elements)."""
    import oracle
    B = np.float32(255.0)
    rng = np.random.default_rng(0)
    r = None
    for cand in rng.uniform(0.5, 2.0, 200000).astype(np.float32):
        if np.float32(cand * np.float32(B / cand)) > B:
            r = cand
            break
    assert r is not None
    over = float(np.float32(r * np.float32(B / r))) - 255.0     # one ulp of 255 = 2^-16
    assert over > 0
    if noise_bits == 24:
        hits = [d for d in range(D) if oracle.noise(seed, 0, 0, d, 24) < over]
    else:
        hits = [d for d in range(D) if oracle.noise(seed, 0, 0, d, 16) >= 1.0 - over]
    assert hits, "no element with extreme enough noise; enlarge D"
    x = np.zeros((1, D), dtype=np.float32)
    x[0, 1::2] = r / 2
    for d in hits:
        x[0, d] = r
        g = d // 256
        if x[0, g * 256:(g + 1) * 256].min() != 0.0:
            x[0, g * 256 + (1 if d % 256 == 0 else 0)] = 0.0
    return x, hits


def overshoot_case_f16(b: int, seed: int = 321, D: int = 1 << 18):
    """As clamp_case, for binary16 input, 16-bit noise and width b: a range r (a binary16 number)
    with fl32(r * fl32(B / r)) one ulp above B = 2^b - 1, the group maximum placed on the elements
    that draw the largest noise, 1 - 2^-16.  Returns (x [1, D] float16, those elements)."""
    import oracle
    B = np.float32((1 << b) - 1)
    cands = np.arange(0x3800, 0x4000, dtype=np.uint16).view(np.float16)      # [0.5, 2)
    c32 = cands.astype(np.float32)
    over = (c32 * (B / c32).astype(np.float32)).astype(np.float32) > B
    if not over.any():
        return None, []
    r = cands[np.flatnonzero(over)[0]]
    hits = [d for d in range(D) if oracle.noise(seed, 0, 0, d, 16) >= 1.0 - 2.0 ** -16]
    assert hits, "no element with the largest noise; enlarge D"
    x = np.zeros((1, D), dtype=np.float16)
    x[0, 1::2] = np.float16(float(r) / 2)
    for d in hits:
        x[0, d] = r
        g = d // 256
        if x[0, g * 256:(g + 1) * 256].min() != 0.0:
            x[0, g * 256 + (1 if d % 256 == 0 else 0)] = 0.0
    return x, hits
