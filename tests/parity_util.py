"""Shared helpers of the parity tests (comparison rules and tolerances)."""
from __future__ import annotations

import numpy as np

# Tolerances of the parity bar: relative error per peer row for binary32 state
# and for bfloat16 state (accumulation is binary32 in both cases).
TOL = {0: 1e-6, 1: 1e-2}
# Storage epsilon (unit roundoff) of the two state types.
EPS = {0: 2.0 ** -24, 1: 2.0 ** -9}
ELEM_FACTOR = 8.0


def assert_state_close(got: np.ndarray, want: np.ndarray, tol: float, what: str = "") -> float:
    """The parity bar: per-row relative L2 error <= tol.  On top of it an
    outlier guard: every element within ELEM_FACTOR * tol * (|want| + rms of
    its row).  The row error is a one-sigma measure of the (storage-rounding)
    noise while the largest of 1e5..1e9 element errors sits 4-6 sigma out, so
    the guard is wider than the bar; a wrong element (an error of order rms) is
    still >= 1e2 (bf16) / 1e5 (fp32) times outside it.  Returns the worst row
    error."""
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
    bound = ELEM_FACTOR * tol * (np.abs(want) + rms[:, None])
    bad = np.abs(got - want) > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements outside {ELEM_FACTOR}*tol*(|x|+rms); first at "
                           f"{tuple(np.argwhere(bad)[0])}")
    return worst


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
