"""Shared plumbing of the GPU parity tests (host<->device copies, comparisons)."""
import numpy as np
import torch

RTOL, ATOL = 1e-5, 1e-6          # fp32 reduced gradients and updated rows (spec tolerance)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def table_to_dev(w: np.ndarray) -> torch.Tensor:
    """float32 array -> fp32 tensor; uint16 array of bf16 bit patterns -> bf16 tensor."""
    if w.dtype == np.float32:
        return dev(w)
    assert w.dtype == np.uint16
    return dev(w.view(np.int16)).view(torch.bfloat16)


def table_to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.float32:
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def exact_f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """For values that are exactly representable in bf16 (the hash initialiser's)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value not exact in bf16"
    return (u >> np.uint32(16)).astype(np.uint16)


def assert_close_f32(got: np.ndarray, want: np.ndarray, what: str) -> None:
    got64, want64 = got.astype(np.float64), want.astype(np.float64)
    err = np.abs(got64 - want64)
    tol = ATOL + RTOL * np.abs(want64)
    bad = err > tol
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} elements off, max err {err.max():.3e}"


def _bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def assert_bf16_within_1ulp(got_bits: np.ndarray, want_bits: np.ndarray, what: str) -> None:
    """bf16 results: at most one bf16 ulp from the oracle's.

    Both sides compute the new weight in fp32 and round it once.  Their fp32 values agree to the
    fp32 tolerance above, so the rounded values are neighbours at worst - except where the update
    cancels the weight almost exactly: there the result is tiny, its own ulp is far finer than the
    fp32 tolerance of the operands it was formed from, and the distance in ulps (or the sign) of
    two correct results can be anything.  Such elements pass when they meet the fp32 tolerance.
    """
    g, w = got_bits.astype(np.int32), want_bits.astype(np.int32)
    same_sign = (g >> 15) == (w >> 15)
    dist = np.abs((g & 0x7FFF) - (w & 0x7FFF))
    # +0 / -0 neighbours: both magnitudes zero
    ok = (same_sign & (dist <= 1)) | (((g & 0x7FFF) == 0) & ((w & 0x7FFF) <= 1)) | (((w & 0x7FFF) == 0) & ((g & 0x7FFF) <= 1))
    if not ok.all():
        bad = np.nonzero(~ok)
        gv, wv = _bf16_bits_to_f64(got_bits[bad]), _bf16_bits_to_f64(want_bits[bad])
        still = np.abs(gv - wv) > ATOL + RTOL * np.abs(wv)
        assert not still.any(), (f"{what}: {int(still.sum())} of {ok.size} bf16 elements beyond 1 ulp and beyond the "
                                 f"fp32 tolerance, e.g. got {gv[still][:4]} want {wv[still][:4]}")


def assert_rows_close(got: np.ndarray, want: np.ndarray, what: str) -> None:
    if want.dtype == np.uint16:
        assert_bf16_within_1ulp(got, want, what)
    else:
        assert_close_f32(got, want, what)
