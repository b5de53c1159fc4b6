"""Tolerance check shared by the GPU parity tests, and a record of how far the GPU path sits
from the bound: every check made with a `case` name stores its worst err / bound ratio under
both forms of the bound; tests/conftest.py writes the record to gpurun_out/parity_margins.json
when the session ends (best effort; nothing reads it back)."""
import numpy as np

MARGINS = {}   # "<case> | <tensor>" -> {"entry": worst err / bound_entry, "row": worst err / bound_row}


def margins(got, want, tol=1e-5):
    """(worst err / bound_entry, worst err / bound_row): bound_entry = tol max(|ref|, rms(tensor)),
    bound_row = tol max(|ref|, rms(tensor), rms(ref row))."""
    got = got.cpu().numpy().astype(np.float64) if hasattr(got, "cpu") else np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    if want.size == 0:
        return 0.0, 0.0
    scale = np.sqrt(np.mean(want ** 2))
    row = np.sqrt(np.mean(want ** 2, axis=-1, keepdims=True)) if want.ndim >= 2 else 0.0
    entry = tol * np.maximum(np.abs(want), scale)
    err = np.abs(got - want)
    with np.errstate(divide="ignore", invalid="ignore"):
        r_entry = np.where(err > 0, err / entry, 0.0).max()
        r_row = np.where(err > 0, err / np.maximum(entry, tol * row), 0.0).max()
    return float(r_entry), float(r_row)


def close(got, want, what, tol=1e-5, row_term=True, case=None):
    """row_term=False: the plain reading |gpu - ref| <= tol max(|ref|, rms(tensor))."""
    got = got.cpu().numpy().astype(np.float64) if hasattr(got, "cpu") else np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    scale = np.sqrt(np.mean(want ** 2)) if want.size else 0.0
    row = np.sqrt(np.mean(want ** 2, axis=-1, keepdims=True)) if (want.ndim >= 2 and row_term) else 0.0
    bound = tol * np.maximum(np.maximum(np.abs(want), scale), row)
    err = np.abs(got - want)
    if case is not None:
        r_entry, r_row = margins(got, want, tol)
        key = f"{case} | {what}"
        old = MARGINS.get(key, {"entry": 0.0, "row": 0.0})
        MARGINS[key] = {"entry": round(max(old["entry"], r_entry), 4), "row": round(max(old["row"], r_row), 4)}
    if not np.all(err <= bound):
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: worst at {i}: got {got[i]!r} want {want[i]!r} "
                             f"(err {err[i]:.3e}, bound {bound[i]:.3e}); "
                             f"{np.count_nonzero(err > bound)} of {err.size} out of tolerance")
