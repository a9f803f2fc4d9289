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


def assert_fold(gpu, ref64, what="", rel=REL_FOLD):
    g, r = float(np.asarray(gpu).reshape(-1)[0]), float(np.asarray(ref64).reshape(-1)[0])
    assert abs(g - r) <= rel * max(abs(r), 1e-30), f"{what}: gpu={g!r} ref={r!r} rel={abs(g - r) / max(abs(r), 1e-30):.3e}"


def assert_ulp(gpu, ref32, ulps, what=""):
    gpu = np.asarray(gpu, dtype=F32)
    ref32 = np.asarray(ref32, dtype=F32)
    tol = ulps * np.spacing(np.abs(ref32)).astype(np.float64)
    err = np.abs(gpu.astype(np.float64) - ref32.astype(np.float64))
    if not np.all(err <= tol):
        i = int(np.argmax(err / np.maximum(tol, 1e-300)))
        raise AssertionError(f"{what}: max error {err.reshape(-1)[i] / np.spacing(abs(ref32.reshape(-1)[i])):.2f} ulp "
                             f"at {i}: gpu={gpu.reshape(-1)[i]!r} ref={ref32.reshape(-1)[i]!r}")


def assert_close(gpu, ref, rel, what="", abs_=0.0):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    err = np.abs(gpu - ref)
    tol = rel * np.abs(ref) + abs_
    if not np.all(err <= tol):
        i = int(np.argmax(err - tol))
        raise AssertionError(f"{what}: element {i}: gpu={gpu.reshape(-1)[i]!r} ref={ref.reshape(-1)[i]!r}")


def assert_segmented(gpu, ref64, terms32, off, what=""):
    """Row-wise and norm-wise bound for y = foldSeg(+)(terms, off)."""
    gpu = np.asarray(gpu, dtype=np.float64)
    ref64 = np.asarray(ref64, dtype=np.float64)
    a = np.abs(np.asarray(terms32, dtype=np.float64))
    cs = np.concatenate([[0.0], np.cumsum(a)])
    scale = cs[off[1:].astype(np.int64)] - cs[off[:-1].astype(np.int64)]
    err = np.abs(gpu - ref64)
    bad = err > REL_FOLD * scale + 1e-30
    if np.any(bad):
        i = int(np.flatnonzero(bad)[0])
        raise AssertionError(f"{what}: row {i}: gpu={gpu[i]!r} ref={ref64[i]!r} scale={scale[i]!r}")
    nrm = float(np.linalg.norm(ref64))
    assert float(np.linalg.norm(gpu - ref64)) <= REL_FOLD * max(nrm, 1e-30), f"{what}: norm-wise bound"
