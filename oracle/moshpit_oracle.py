"""ctypes front end of the fp64 CPU oracle (``moshpit_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module
and this module never imports the product package.

The arithmetic lives in the C file; this module only marshals numpy arrays and,
for large states, hands independent column slabs to worker threads (columns
never interact in an averaging round: the argument of App. C.2 is
component-wise).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moshpit_oracle.c")
_LIB = os.path.join(_HERE, "libmoshpit_oracle.so")

_i64, _i32, _u64, _f64 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_double
_ptr = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no vector intrinsics, strict fp)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off",
             "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # MOSHPIT_ORACLE_LIB: another build of moshpit_oracle.c to load instead (the
        # sanitizer test points it at an ASan/UBSan build of the same source)
        lib = ctypes.CDLL(os.environ.get("MOSHPIT_ORACLE_LIB") or build())
        lib.oracle_digits.argtypes = [_i64, _i32, _i32, _ptr]
        lib.oracle_digits.restype = None
        lib.oracle_group_keys.argtypes = [_i64, _i32, _i32, _i64, _ptr]
        lib.oracle_group_ids.argtypes = [_i64, _i32, _i32, _i64, _ptr]
        lib.oracle_round.argtypes = [_ptr, _i64, _i64, _i64, _i32, _i32, _i64, _ptr]
        lib.oracle_quantize.argtypes = [_ptr, _i64, _i64, _i64, _i32]
        lib.oracle_dist_to_mean.argtypes = [_ptr, _i64, _i64, _i64]
        lib.oracle_dist_to_mean.restype = _f64
        lib.oracle_dist_to_mean_subset.argtypes = [_ptr, _i64, _i64, _i64, _ptr]
        lib.oracle_dist_to_mean_subset.restype = _f64
        lib.oracle_schedule_masks.argtypes = [_i32, _f64, _u64, _i32, _i64, _i64, _i32, _ptr]
        lib.oracle_dynamic_init.argtypes = [_i64, _i32, _i32, _ptr]
        lib.oracle_dynamic_round.argtypes = [_ptr, _i64, _i64, _i64, _i32, _i32, _ptr, _u64, _i64, _ptr]
        lib.oracle_local_step.argtypes = [_ptr, _ptr, _i64, _i64, _i64, _i64, _f64, _ptr]
        lib.oracle_sgd_round.argtypes = [_ptr, _ptr, _i64, _i64, _i64, _i64, _f64, _i32, _i32, _i64, _ptr]
        lib.oracle_skip_filter.argtypes = [_i64, _i32, _i32, _i64, _ptr, _ptr]
        lib.oracle_refresh_donors.argtypes = [_i64, _ptr, _ptr, _u64, _i64, _ptr]
        lib.oracle_refresh.argtypes = [_ptr, _i64, _i64, _i64, _ptr]
        lib.oracle_random_permutation.argtypes = [_u64, _i64, _i64, _ptr]
        lib.oracle_grouped_round.argtypes = [_ptr, _i64, _i64, _i64, _ptr, _i64, _i32, _ptr]
        lib.oracle_random_groups_round.argtypes = [_ptr, _i64, _i64, _i64, _u64, _i64, _i32, _ptr]
        lib.oracle_run.argtypes = [_ptr, _i64, _i64, _i64, _i32, _i32, _i64, _i32, _ptr, _i32, _ptr]
        _lib = lib
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def _state(X: np.ndarray) -> np.ndarray:
    if X.dtype != np.float64 or X.ndim != 2 or X.strides[1] != 8 or X.strides[0] % 8:
        raise TypeError("oracle state must be a 2-D float64 array with unit column stride")
    return X


def _mask_ptr(alive, N):
    if alive is None:
        return None, None
    a = np.ascontiguousarray(alive, dtype=np.uint8)
    if a.shape != (N,):
        raise ValueError("alive mask must have shape (N,)")
    return a, a.ctypes.data


def digits(i: int, M: int, d: int) -> list[int]:
    out = np.zeros(d, dtype=np.int32)
    _load().oracle_digits(i, M, d, out.ctypes.data)
    return out.tolist()


def group_keys(N: int, M: int, d: int, t: int) -> np.ndarray:
    keys = np.empty(N, dtype=np.int32)
    _check(_load().oracle_group_keys(N, M, d, t, keys.ctypes.data), "group_keys")
    return keys


def group_ids(N: int, M: int, d: int, t: int) -> np.ndarray:
    gid = np.empty(N, dtype=np.int64)
    _check(_load().oracle_group_ids(N, M, d, t, gid.ctypes.data), "group_ids")
    return gid


def round_(X: np.ndarray, M: int, d: int, t: int, alive=None) -> None:
    """One averaging round, in place, on a float64 [N, W] array (or view)."""
    X = _state(X)
    N, W = X.shape
    keep, ptr = _mask_ptr(alive, N)
    _check(_load().oracle_round(X.ctypes.data, N, W, X.strides[0] // 8, M, d, t, ptr), "round")


def quantize(X: np.ndarray, dtype: int) -> None:
    X = _state(X)
    N, W = X.shape
    _check(_load().oracle_quantize(X.ctypes.data, N, W, X.strides[0] // 8, dtype), "quantize")


def dist_to_mean(X: np.ndarray) -> float:
    X = _state(X)
    N, W = X.shape
    return float(_load().oracle_dist_to_mean(X.ctypes.data, N, W, X.strides[0] // 8))


def dist_to_mean_subset(X: np.ndarray, present=None) -> float:
    """Average distortion over the rows with present != 0 (None = all rows)."""
    X = _state(X)
    N, W = X.shape
    keep, ptr = _mask_ptr(present, N)
    return float(_load().oracle_dist_to_mean_subset(X.ctypes.data, N, W, X.strides[0] // 8, ptr))


def schedule_masks(kind: int, p: float, seed: int, down: int, N: int, t0: int, rounds: int) -> np.ndarray:
    """uint8 [rounds, N], 1 = alive, for rounds t0..t0+rounds-1."""
    masks = np.empty((rounds, N), dtype=np.uint8)
    _check(_load().oracle_schedule_masks(kind, float(p), seed, down, N, t0, rounds,
                                         masks.ctypes.data), "schedule_masks")
    return masks


def dynamic_init(N: int, M: int, d: int) -> np.ndarray:
    """Initial chunk-index keys (Eq. 2): int32 [N, d-1]."""
    keys = np.zeros((N, max(d - 1, 0)), dtype=np.int32)
    _check(_load().oracle_dynamic_init(N, M, d, keys.ctypes.data), "dynamic_init")
    return keys


def dynamic_round(X: np.ndarray, M: int, d: int, keys: np.ndarray, seed: int, t: int, alive=None) -> None:
    """One round of Alg. 1 with chunk-index keys; X and keys are updated in place."""
    X = _state(X)
    N, W = X.shape
    assert keys.dtype == np.int32 and keys.shape == (N, max(d - 1, 0)) and keys.flags.c_contiguous
    keep, ptr = _mask_ptr(alive, N)
    _check(_load().oracle_dynamic_round(X.ctypes.data, N, W, X.strides[0] // 8, M, d, keys.ctypes.data, seed, t, ptr),
           "dynamic_round")


def local_step(X: np.ndarray, G: np.ndarray, gamma: float, alive=None) -> None:
    """theta_i <- theta_i - gamma * g_i for the peers that take part (Alg. 2, local iteration)."""
    X, G = _state(X), _state(G)
    N, W = X.shape
    assert G.shape == X.shape
    keep, ptr = _mask_ptr(alive, N)
    _check(_load().oracle_local_step(X.ctypes.data, G.ctypes.data, N, W, X.strides[0] // 8, G.strides[0] // 8,
                                     float(gamma), ptr), "local_step")


def sgd_round(X: np.ndarray, G: np.ndarray, gamma: float, M: int, d: int, t: int, alive=None) -> None:
    """theta_i <- group average of (theta_j - gamma * g_j) (Alg. 2, communication iteration)."""
    X, G = _state(X), _state(G)
    N, W = X.shape
    assert G.shape == X.shape
    keep, ptr = _mask_ptr(alive, N)
    _check(_load().oracle_sgd_round(X.ctypes.data, G.ctypes.data, N, W, X.strides[0] // 8, G.strides[0] // 8,
                                    float(gamma), M, d, t, ptr), "sgd_round")


def skip_filter(N: int, M: int, d: int, t: int, alive) -> np.ndarray:
    """Masks of the group-skip behaviour: a group with a failed member sits the round out."""
    a = np.ascontiguousarray(alive, dtype=np.uint8)
    out = np.empty(N, dtype=np.uint8)
    _check(_load().oracle_skip_filter(N, M, d, t, a.ctypes.data, out.ctypes.data), "skip_filter")
    return out


def refresh_donors(prev, cur, seed: int, t: int) -> np.ndarray:
    """donor[i] >= 0 for every peer that returns in round t (present now, absent in round t-1):
    the up-to-date peer whose parameters it takes; -1 elsewhere."""
    a = np.ascontiguousarray(prev, dtype=np.uint8)
    b = np.ascontiguousarray(cur, dtype=np.uint8)
    if a.shape != b.shape or a.ndim != 1:
        raise ValueError("masks must be two vectors of the same length")
    donor = np.empty(a.shape[0], dtype=np.int32)
    _check(_load().oracle_refresh_donors(a.shape[0], a.ctypes.data, b.ctypes.data, seed, t, donor.ctypes.data),
           "refresh_donors")
    return donor


def refresh(X: np.ndarray, donor) -> None:
    """X[i] <- X[donor[i]] wherever donor[i] >= 0."""
    X = _state(X)
    N, W = X.shape
    dn = np.ascontiguousarray(donor, dtype=np.int32)
    if dn.shape != (N,):
        raise ValueError("donor must have shape (N,)")
    _check(_load().oracle_refresh(X.ctypes.data, N, W, X.strides[0] // 8, dn.ctypes.data), "refresh")


def random_permutation(seed: int, t: int, N: int) -> np.ndarray:
    perm = np.empty(N, dtype=np.int64)
    _check(_load().oracle_random_permutation(seed, t, N, perm.ctypes.data), "random_permutation")
    return perm


def grouped_round(X: np.ndarray, index, group_size: int, alive=None) -> None:
    """Average consecutive chunks of `group_size` entries of the peer list `index`."""
    X = _state(X)
    N, W = X.shape
    idx = np.ascontiguousarray(index, dtype=np.int64)
    keep, ptr = _mask_ptr(alive, N)
    _check(_load().oracle_grouped_round(X.ctypes.data, N, W, X.strides[0] // 8, idx.ctypes.data, len(idx),
                                        group_size, ptr), "grouped_round")


def random_groups_round(X: np.ndarray, seed: int, t: int, group_size: int, alive=None) -> None:
    X = _state(X)
    N, W = X.shape
    keep, ptr = _mask_ptr(alive, N)
    _check(_load().oracle_random_groups_round(X.ctypes.data, N, W, X.strides[0] // 8, seed, t, group_size, ptr),
           "random_groups_round")


def run(X: np.ndarray, M: int, d: int, t0: int, rounds: int, masks=None,
        quantize_dtype: int = -1, want_dist: bool = False, threads: int = 1,
        slab: int = 4096):
    """Rounds t0..t0+rounds-1 in place.  Returns the rounds+1 distortions when asked.

    ``threads`` > 1 splits the columns into slabs of ``slab`` columns and runs
    the (single-threaded) C oracle on each slab in a worker thread.
    """
    X = _state(X)
    N, W = X.shape
    lib = _load()
    mptr = None
    if masks is not None:
        masks = np.ascontiguousarray(masks, dtype=np.uint8)
        if masks.shape != (rounds, N):
            raise ValueError("masks must have shape (rounds, N)")
        mptr = masks.ctypes.data
    ld = X.strides[0] // 8

    def one(c0: int):
        w = min(slab, W - c0)
        dist = np.zeros(rounds + 1, dtype=np.float64) if want_dist else None
        rc = lib.oracle_run(X.ctypes.data + 8 * c0, N, w, ld, M, d, t0, rounds, mptr,
                            quantize_dtype, dist.ctypes.data if want_dist else None)
        _check(rc, "run")
        return dist

    starts = list(range(0, W, slab)) if W > 0 else []
    if threads <= 1 or len(starts) <= 1:
        parts = [one(c0) for c0 in starts]
    else:
        with ThreadPoolExecutor(max_workers=threads) as pool:
            parts = list(pool.map(one, starts))
    if want_dist:
        total = np.zeros(rounds + 1, dtype=np.float64)
        for part in parts:
            total += part
        return total
    return None
