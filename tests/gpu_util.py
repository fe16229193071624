"""Helpers for the GPU parity tests: host <-> device marshalling and the comparison rules.

Tolerances (binary32 path against the binary64-reduction oracle):
  coefficients   |d| <= 1e-4 * max_i |coef_i|                per vector
  y, h, c        |d| <= 1e-4 * |ref| + 1e-4 * rms(ref row)   per element
  packed codes   bit-exact; a differing bit is accepted only if its entry sits within
                 1e-5 * max|v| of an interval boundary of the oracle's code table (a
                 binary32 near-tie), and such flips are counted and reported.
"""
import numpy as np
import torch

import oracle

DEV = "cuda:0"


def to_dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(DEV)


def planes_host(t):
    return t.cpu().numpy().view(np.uint32)


def host(t):
    return t.cpu().numpy()


def assert_coef_close(got, ref, what="coef"):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    bad = ~(np.abs(got - ref) <= 1e-4 * scale + 1e-30)   # (NaN counts as a mismatch)
    assert not bad.any(), "%s: %d mismatches, worst %g" % (what, bad.sum(), np.abs(got - ref).max())


def assert_vec_close(got, ref, what="y"):
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    tol = 1e-4 * np.abs(ref) + 1e-4 * rms + 1e-30
    bad = ~(np.abs(got - ref) <= tol)   # (NaN counts as a mismatch)
    assert not bad.any(), "%s: %d mismatches, worst ratio %g" % (what, bad.sum(), (np.abs(got - ref) / tol).max())


def worst_ratio(got, ref):
    """Largest |got - ref| in units of the tolerance of assert_vec_close (1.0 = at the bar)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    rms = np.sqrt((ref ** 2).mean(axis=-1, keepdims=True))
    tol = 1e-4 * np.abs(ref) + 1e-4 * rms + 1e-30
    return float((np.abs(got - ref) / tol).max())


def unpack_bits(planes, n):
    k, rows, wpr = planes.shape
    b = np.unpackbits(np.ascontiguousarray(planes).view(np.uint8).reshape(k, rows, wpr * 4), axis=2,
                      bitorder="little")
    return b[:, :, :n]


def compare_codes(X, planes_gpu, planes_ref, coef_ref):
    """Bit-exact comparison with near-tie accounting.  Returns (flipped_entries, rows_with_flips).

    Pad bits must be zero.  A differing entry must be a binary32 near-tie at a boundary of the
    code table built from the oracle's coefficients of that row."""
    X = np.asarray(X, np.float32)
    rows, n = X.shape
    k = planes_ref.shape[0]
    wpr = planes_ref.shape[2]
    assert planes_gpu.shape == planes_ref.shape
    full = np.unpackbits(np.ascontiguousarray(planes_gpu).view(np.uint8).reshape(k, rows, wpr * 4), axis=2,
                         bitorder="little")
    assert not full[:, :, n:].any(), "pad bits must be zero"
    if np.array_equal(planes_gpu, planes_ref):
        return 0, 0
    diff = (unpack_bits(planes_gpu, n) != unpack_bits(planes_ref, n)).any(axis=0)   # [rows, n]
    flipped_rows = np.nonzero(diff.any(axis=1))[0]
    total = 0
    for r in flipped_rows:
        v, pat, mid = oracle.code_table(coef_ref[r])
        tol = 1e-5 * np.abs(v).max()
        for l in np.nonzero(diff[r])[0]:
            d = np.abs(mid.astype(np.float64) - float(X[r, l])).min()
            assert d <= tol, "row %d entry %d differs and is not a near-tie (distance %g, tol %g)" % (r, l, d, tol)
            total += 1
    return total, len(flipped_rows)
