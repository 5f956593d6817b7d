"""The parity bars, in one place for the tests and for bench.py's in-run check (comparisons only).

fp32 results (reduced gradients, Adagrad state, updated rows): |got - want| <= 1e-6 + 1e-5 * |want| per element.
bf16 rows: at most one bf16 ulp between the two 16-bit patterns; the only exception is derived below and is
counted, so that it cannot quietly become the rule.
"""
from __future__ import annotations

import numpy as np

RTOL, ATOL = 1e-5, 1e-6
BF16_FALLBACK_SHARE = 1e-6      # share of the elements of one comparison that may take the exception below ...
BF16_FALLBACK_FLOOR = 2         # ... or this many, whichever is more (a small array has no millionth)


def assert_close_f32(got: np.ndarray, want: np.ndarray, what: str) -> None:
    got64, want64 = got.astype(np.float64), want.astype(np.float64)
    err = np.abs(got64 - want64)
    tol = ATOL + RTOL * np.abs(want64)
    bad = err > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} elements off, max err {err.max():.3e}"


def _bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def bf16_beyond_1ulp(got_bits: np.ndarray, want_bits: np.ndarray) -> np.ndarray:
    """Boolean mask of the elements whose 16-bit patterns are more than one ulp apart."""
    g, w = got_bits.astype(np.int32), want_bits.astype(np.int32)
    same_sign = (g >> 15) == (w >> 15)
    dist = np.abs((g & 0x7FFF) - (w & 0x7FFF))
    # +0 / -0 neighbours: both magnitudes zero or one
    ok = (same_sign & (dist <= 1)) | (((g & 0x7FFF) == 0) & ((w & 0x7FFF) <= 1)) | (((w & 0x7FFF) == 0) & ((g & 0x7FFF) <= 1))
    return ~ok


def assert_bf16_within_1ulp(got_bits: np.ndarray, want_bits: np.ndarray, what: str) -> int:
    """bf16 results: at most one bf16 ulp from the oracle's.  Returns the number of elements that took the
    exception.

    Both sides compute the new weight in fp32 and round it once.  Their fp32 values agree to the fp32
    tolerance above, so the rounded values are neighbours at worst - except where the update cancels the
    weight almost exactly: there the result is tiny, its own ulp is far finer than the fp32 tolerance of the
    operands it was formed from, and the distance in ulps (or the sign) of two correct results can be
    anything.  Such elements pass when they meet the fp32 tolerance, and there may be at most
    max(BF16_FALLBACK_FLOOR, BF16_FALLBACK_SHARE * elements) of them in one comparison.
    """
    beyond = bf16_beyond_1ulp(got_bits, want_bits)
    n_beyond = int(beyond.sum())
    if n_beyond:
        gv, wv = _bf16_bits_to_f64(got_bits[beyond]), _bf16_bits_to_f64(want_bits[beyond])
        still = np.abs(gv - wv) > ATOL + RTOL * np.abs(wv)
        assert not still.any(), (f"{what}: {int(still.sum())} of {beyond.size} bf16 elements beyond 1 ulp and beyond the "
                                 f"fp32 tolerance, e.g. got {gv[still][:4]} want {wv[still][:4]}")
        allowed = max(BF16_FALLBACK_FLOOR, int(BF16_FALLBACK_SHARE * beyond.size))
        assert n_beyond <= allowed, (f"{what}: {n_beyond} of {beyond.size} bf16 elements are beyond 1 ulp (inside the "
                                     f"fp32 tolerance); at most {allowed} may be")
    return n_beyond


def assert_rows_close(got: np.ndarray, want: np.ndarray, what: str) -> None:
    """uint16 arrays are bf16 bit patterns, float32 arrays fp32 values."""
    if want.dtype == np.uint16:
        assert_bf16_within_1ulp(got, want, what)
    else:
        assert_close_f32(got, want, what)
