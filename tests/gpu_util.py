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
