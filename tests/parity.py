"""Comparison rules between the HIP path and the CPU oracle.

  * integer / index arrays and fp32 arrays computed with + - * only: bit-exact
  * fp32 reductions: |gpu - ref64| <= 1e-5 * max(|ref64|, tiny)   (the stated bound)
  * segmented (+) folds: row-wise |gpu - ref64| <= 1e-5 * sum_k |term_k| (the scale
    of a row's summation error; a row that cancels to ~0 has no meaningful relative
    error) and norm-wise ||gpu - ref||_2 <= 1e-5 ||ref||_2
  * sin / exp based maps: the oracle rounds the fp64 value once; the device
    function must stay within 4 ulp of it
  * arrays downstream of those maps: relative 1e-6 plus the propagated ulps
    (stated per call site)
  * values that are not finite are compared by class, never by subtraction: a NaN
    must meet a NaN, an infinity the infinity of the same sign, and the bounds
    above apply to the remaining (finite) elements
"""
import numpy as np

F32 = np.float32
REL_FOLD = 1e-5


def assert_bit_exact(gpu, ref, what=""):
    gpu, ref = np.asarray(gpu), np.asarray(ref)
    assert gpu.shape == ref.shape, f"{what}: shape {gpu.shape} vs {ref.shape}"
    if gpu.dtype.kind == "f":
        same = gpu.view(np.int32) == ref.astype(F32).view(np.int32)
    else:
        same = gpu == ref
    if not np.all(same):
        bad = np.flatnonzero(~same.reshape(-1))
        i = int(bad[0])
        raise AssertionError(f"{what}: {bad.size} of {gpu.size} elements differ; first at {i}: "
                             f"gpu={gpu.reshape(-1)[i]!r} ref={ref.reshape(-1)[i]!r}")


def same_class(gpu, ref, what=""):
    """Checks that NaNs meet NaNs and infinities meet infinities of the same sign; returns the
    mask of the elements that are finite on the reference side (and therefore on both)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    for name, g, r in (("NaN", np.isnan(gpu), np.isnan(ref)), ("+inf", gpu == np.inf, ref == np.inf),
                       ("-inf", gpu == -np.inf, ref == -np.inf)):
        if not np.array_equal(g, r):
            i = int(np.flatnonzero((g != r).reshape(-1))[0])
            raise AssertionError(f"{what}: element {i}: gpu={gpu.reshape(-1)[i]!r} ref={ref.reshape(-1)[i]!r} ({name} on one side only)")
    return np.isfinite(ref)


def assert_fold(gpu, ref64, what="", rel=REL_FOLD):
    g, r = float(np.asarray(gpu).reshape(-1)[0]), float(np.asarray(ref64).reshape(-1)[0])
    if not same_class([g], [r], what)[0]:
        return
    assert abs(g - r) <= rel * max(abs(r), 1e-30), f"{what}: gpu={g!r} ref={r!r} rel={abs(g - r) / max(abs(r), 1e-30):.3e}"


def assert_ulp(gpu, ref32, ulps, what=""):
    gpu = np.asarray(gpu, dtype=F32)
    ref32 = np.asarray(ref32, dtype=F32)
    finite = same_class(gpu, ref32, what)
    gpu, ref32 = np.where(finite, gpu, F32(0)), np.where(finite, ref32, F32(0))
    tol = ulps * np.spacing(np.abs(ref32)).astype(np.float64)
    err = np.abs(gpu.astype(np.float64) - ref32.astype(np.float64))
    if not np.all(err <= tol):
        i = int(np.argmax(err / np.maximum(tol, 1e-300)))
        raise AssertionError(f"{what}: max error {err.reshape(-1)[i] / np.spacing(abs(ref32.reshape(-1)[i])):.2f} ulp "
                             f"at {i}: gpu={gpu.reshape(-1)[i]!r} ref={ref32.reshape(-1)[i]!r}")


def assert_close(gpu, ref, rel, what="", abs_=0.0):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    finite = same_class(gpu, ref, what)
    gpu, ref = np.where(finite, gpu, 0.0), np.where(finite, ref, 0.0)
    err = np.abs(gpu - ref)
    tol = rel * np.abs(ref) + abs_
    if not np.all(err <= tol):
        i = int(np.argmax(err - tol))
        raise AssertionError(f"{what}: element {i}: gpu={gpu.reshape(-1)[i]!r} ref={ref.reshape(-1)[i]!r}")


def assert_segmented(gpu, ref64, terms32, off, what=""):
    """Row-wise and norm-wise bound for y = foldSeg(+)(terms, off)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref64 = np.asarray(ref64, dtype=np.float64)
    finite = same_class(gpu, ref64, what)          # a row with a term that is not finite is not finite itself
    gpu, ref64 = np.where(finite, gpu, 0.0), np.where(finite, ref64, 0.0)
    a = np.abs(np.asarray(terms32, dtype=np.float64))
    a = np.where(np.isfinite(a), a, 0.0)
    cs = np.concatenate([[0.0], np.cumsum(a)])
    scale = cs[off[1:].astype(np.int64)] - cs[off[:-1].astype(np.int64)]
    err = np.abs(gpu - ref64)
    bad = err > REL_FOLD * scale + 1e-30
    if np.any(bad):
        i = int(np.flatnonzero(bad)[0])
        raise AssertionError(f"{what}: row {i}: gpu={gpu[i]!r} ref={ref64[i]!r} scale={scale[i]!r}")
    nrm = float(np.linalg.norm(ref64))
    assert float(np.linalg.norm(gpu - ref64)) <= REL_FOLD * max(nrm, 1e-30), f"{what}: norm-wise bound"
