"""Shared helpers of the parity tests (comparison rules and tolerances)."""
from __future__ import annotations

import numpy as np

# Tolerances of the parity bar: relative error per peer row for binary32 state
# and for bfloat16 state (accumulation is binary32 in both cases).
TOL = {0: 1e-6, 1: 1e-2}
# Storage epsilon (unit roundoff) of the two state types.
EPS = {0: 2.0 ** -24, 1: 2.0 ** -9}
# Width of the element-wise outlier guard in units of tol, per storage type.  binary32: the
# guard IS the tolerance (worst element errors measured on the GPU stay below 0.3 * tol).
# bfloat16: the row error is a one-sigma measure of the storage-rounding noise (unit roundoff
# 2^-9 against tol 1e-2) while the largest of 1e5..1e9 element errors sits 4-6 sigma out.
ELEM_FACTOR = {0: 1.0, 1: 8.0}


def assert_state_close(got: np.ndarray, want: np.ndarray, tol: float, what: str = "") -> float:
    """The parity bar: per-row relative L2 error <= tol.  On top of it an
    outlier guard: every element within ELEM_FACTOR * tol * (|want| + rms of
    its row), the factor being 1 for the binary32 tolerance and 8 for the
    bfloat16 one; a wrong element (an error of order rms) is >= 1e2 (bf16) /
    1e6 (fp32) times outside it.  Returns the worst row error."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape
    if want.size == 0:
        return 0.0
    norm = np.linalg.norm(want, axis=1)
    err = np.linalg.norm(got - want, axis=1)
    rel = np.where(norm > 0, err / np.where(norm > 0, norm, 1.0), err)
    worst = float(rel.max())
    assert worst <= tol, f"{what}: worst row relative error {worst:.3e} > {tol:.1e} (row {int(rel.argmax())})"
    rms = norm / np.sqrt(want.shape[1])
    factor = ELEM_FACTOR[1] if tol >= 1e-3 else ELEM_FACTOR[0]
    bound = factor * tol * (np.abs(want) + rms[:, None])
    err_el = np.abs(got - want)
    bad = err_el > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements outside {factor}*tol*(|x|+rms); first at "
                           f"{tuple(np.argwhere(bad)[0])}, worst ratio {float((err_el / bound).max()):.3f}")
    return worst


def worst_element_ratio(got: np.ndarray, want: np.ndarray, tol: float) -> float:
    """Largest element error in units of tol * (|want| + rms of its row)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = np.linalg.norm(want, axis=1) / np.sqrt(want.shape[1])
    return float((np.abs(got - want) / (tol * (np.abs(want) + rms[:, None]) + 1e-300)).max())


def assert_dist_close(got, want, tol: float, floor: float, what: str = "") -> None:
    """Distortion values: |got - want| <= tol * want + floor.  The floor covers
    the converged regime, where the fp64 oracle is ~0 and the stored state
    carries its own rounding noise."""
    got = np.atleast_1d(np.asarray(got, dtype=np.float64))
    want = np.atleast_1d(np.asarray(want, dtype=np.float64))
    assert got.shape == want.shape
    bad = np.abs(got - want) > tol * np.abs(want) + floor
    assert not bad.any(), f"{what}: dist mismatch got={got} want={want} floor={floor:.3e}"


def dist_floor(P: int, dtype: int, rms0: float) -> float:
    """Rounding-noise floor of the distortion of a state stored in `dtype`
    whose entries have magnitude ~rms0: P * (eps * rms0)^2, with a safety
    factor of 4."""
    return 4.0 * P * (EPS[dtype] * rms0) ** 2


def sample_columns(P: int, count: int, seed: int, tile: int = 2048) -> np.ndarray:
    """Column indices that cover the first and last tiles, tile boundaries and
    the ragged tail, plus random ones; sorted and unique."""
    rng = np.random.default_rng(seed)
    cols = set(range(min(P, 16))) | set(range(max(0, P - 16), P))
    for b in (tile, 2 * tile, (P // tile) * tile, (P // 2 // tile) * tile):
        cols |= {c for c in range(b - 4, b + 4) if 0 <= c < P}
    need = max(0, count - len(cols))
    cols |= set(rng.integers(0, P, size=need).tolist())
    return np.array(sorted(cols), dtype=np.int64)
