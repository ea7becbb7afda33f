"""The 16-bit rounding rule, code = floor(fl32(u + noise)), enumerated over every one of the 65,536
noise values for chosen scaled values u (Sec. 4.1: stochastic rounding should return ceil(u) with
probability frac(u); Thm. 1 builds on that).  The single binary32 addition rounds, so the
probability of rounding up is frac(u) only up to the noise grid: the bound pinned here is
|P(up) - frac(u)| <= 2^-16, together with code <= B, grid points never moving, and the decision
being monotone in the noise.

u is controlled exactly: a group with minimum 0 and maximum B has range B, factor B / B = 1 and
therefore u = x.  The noise of every element comes from the oracle's own generator
(`oracle.noise`), which the Philox pins tie to the published vectors and to rocRAND.
"""
import numpy as np
import pytest

import oracle

D = 1 << 21          # 2M elements: every 16-bit noise value occurs (a value is missed with probability e^-32)
SEED, TAG = 77, 3
_noise_cache = {}


def _noise_index():
    """k[d] = noise of element d times 2^16, as an integer."""
    if "k" not in _noise_cache:
        k = np.empty(D, dtype=np.int64)
        L = oracle.lib()
        for d in range(D):
            k[d] = int(round(L.orc_noise(SEED, TAG, 0, d, 16) * 65536.0))
        lead = (np.arange(D) % 256) < 2                  # per group: element 0 is the minimum, element 1 the maximum
        kk = k[~lead]
        order = np.argsort(kk, kind="stable")
        ks = kk[order]
        starts = np.searchsorted(ks, np.arange(65536), side="left")
        ends = np.searchsorted(ks, np.arange(65536), side="right")
        _noise_cache.update(k=k, lead=lead, order=order, starts=starts, present=ends > starts)
    return _noise_cache


def _cases():
    for b in range(1, 9):
        B = (1 << b) - 1
        us = [0.0, float(B), 0.5, np.float32(0.5) - np.float32(2.0 ** -26), np.float32(2.0 ** -20),
              np.float32(1.0) - np.float32(2.0 ** -24), np.float32(0.3), np.float32(1 / 3),
              np.float32(B) - np.float32(2.0 ** -10), np.nextafter(np.float32(B), np.float32(0)),
              np.float32(B) - np.float32(2.0 ** -16), np.float32(B - 1) + np.float32(2.0 ** -18) if B > 1 else np.float32(2.0 ** -18),
              np.float32(B - 0.5) + np.float32(2.0 ** -21)]
        if B >= 2:
            us += [np.float32(1.0) + np.float32(2.0 ** -20), np.float32(2.0) - np.float32(2.0 ** -22)]
        for u in us:
            yield b, np.float32(u)


@pytest.mark.parametrize("b", range(1, 9))
def test_probability_of_rounding_up_is_within_one_grid_step_of_the_fraction(b):
    cache = _noise_index()
    k, lead, order, starts, present = (cache[n] for n in ("k", "lead", "order", "starts", "present"))
    assert k.min() == 0 and k.max() == 65535
    assert present.sum() >= 65530                            # elements 0, 1 of each group are left out
    B = (1 << b) - 1
    bits = np.array([b], dtype=np.uint8)
    for bb, u in _cases():
        if bb != b:
            continue
        assert 0.0 <= float(u) <= B
        x = np.full((1, D), u, dtype=np.float32)
        x[0, 0::256] = 0.0
        x[0, 1::256] = B
        codes = oracle.quantize_codes(x, bits, SEED, TAG, noise_bits=16)[0].astype(np.int64)
        assert codes.max() <= B and codes.min() >= 0
        assert np.all(codes[0::256] == 0) and np.all(codes[1::256] == B)      # grid points keep their code
        c = codes[~lead]
        fl = int(np.floor(float(u)))
        frac = float(u) - fl                                                   # exact in double
        up = c - fl
        assert set(np.unique(up)) <= {0, 1}
        # the decision is a function of the noise value alone, and monotone in it
        ups = up[order]
        lo = np.minimum.reduceat(ups, starts[present])
        hi = np.maximum.reduceat(ups, starts[present])
        assert np.array_equal(lo, hi), "two elements with the same noise got different decisions"
        decision = lo                                                          # per present noise value, ascending
        assert np.all(np.diff(decision) >= 0), "rounding up must be monotone in the noise"
        # P(up) over the 65,536 equally likely noise values; missing values (at most six) count either way
        ups_count = int(decision.sum())
        missing = 65536 - int(present.sum())
        p_lo, p_hi = ups_count / 65536.0, (ups_count + missing) / 65536.0
        assert p_lo - 2.0 ** -16 <= frac <= p_hi + 2.0 ** -16, (b, float(u), p_lo, p_hi, frac)
        if frac == 0.0:
            assert ups_count == 0                                              # an integer u never moves
