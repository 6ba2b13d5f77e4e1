"""Helpers for the GPU parity tests: tolerances of the benchmark spec and device/host shuttling."""
import numpy as np

REL32, ABS32 = 1e-4, 1e-5     # fp32 results
REL_BF16 = 2e-2               # bf16 GEMM-derived results, relative to max(|ref|, RMS(ref))


def to_np(t):
    import torch
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


def dev(a, dtype=None):
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def assert_close32(got, ref, what, rel=REL32, abs_=ABS32, mask=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    err = np.abs(got - ref)
    tol = abs_ + rel * np.abs(ref)
    bad = ~(err <= tol)
    if mask is not None:
        bad &= mask
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, err - tol, -np.inf)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside rel {rel} / abs {abs_}; worst at {i}: "
                             f"got {got[i]!r} ref {ref[i]!r}")


def assert_close_bf16(got, ref, what, rel=REL_BF16, mask=None):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    sel = ref if mask is None else ref[mask]
    rms = float(np.sqrt(np.mean(sel ** 2))) if sel.size else 0.0
    err = np.abs(got - ref)
    tol = rel * np.maximum(np.abs(ref), rms) + 1e-30
    bad = ~(err <= tol)
    if mask is not None:
        bad &= mask
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, err / tol, -np.inf)), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} outside {rel} * max(|ref|, rms={rms:.3g}); "
                             f"worst at {i}: got {got[i]!r} ref {ref[i]!r}")


def rel_rms_err(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.sqrt(np.mean((got - ref) ** 2)) / max(np.sqrt(np.mean(ref ** 2)), 1e-300))


def bf16_chain_report(got, ref, rel=REL_BF16):
    """(fraction of elements outside rel * max(|ref|, rms), worst error in units of that band, relative RMS error)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
    band = rel * np.maximum(np.abs(ref), rms) + 1e-30
    ratio = np.abs(got - ref) / band
    return float(np.mean(ratio > 1.0)), float(ratio.max()), rel_rms_err(got, ref)


def assert_close_bf16_chain(got, ref, what, rel=REL_BF16, outliers=1e-3, wide=3.0, rms=1e-2):
    """For results at the end of a chain of bf16 products (hypernet gradients behind four re-rounded layers and the
    factor products): the relative RMS error stays below `rms`, all but a fraction `outliers` of the elements sit
    inside the band of a single bf16 GEMM output, rel * max(|ref|, RMS(ref)), and none leaves `wide` times that
    band.  A wrong result (a dropped term, a transposed operand, a missing factor) misses all three by far."""
    frac, worst, r = bf16_chain_report(got, ref, rel)
    assert r < rms, f"{what}: relative RMS error {r:.4g} >= {rms}"
    assert frac <= outliers, f"{what}: {frac:.2e} of the elements outside {rel} * max(|ref|, rms)"
    assert worst <= wide, f"{what}: worst element {worst:.2f} bands away"
