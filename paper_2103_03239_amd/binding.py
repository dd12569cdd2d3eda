"""Thin ctypes binding of libmoshpit.so (see include/moshpit.h).

Argument marshalling only: every step of a round runs in the library's HIP
kernels.  PyTorch supplies device memory (the state tensor) and the stream.
There is no fallback: if the library is missing or a call fails, an exception
is raised.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoshpit.so")

F32, BF16 = 0, 1
SCHED_NONE, SCHED_IID, SCHED_REJOIN, SCHED_EXPLICIT = 0, 1, 2, 3
RUN_DEFAULT, RUN_FUSED = 0, 1

EXPORTS = [
    "moshpit_create", "moshpit_destroy", "moshpit_bind_state", "moshpit_round", "moshpit_round_dev",
    "moshpit_run", "moshpit_dist_to_mean", "moshpit_dist_to_mean_static", "moshpit_dist_to_mean_subset", "moshpit_group_keys", "moshpit_schedule_mask",
    "moshpit_dynamic_reset", "moshpit_dynamic_round", "moshpit_dynamic_keys", "moshpit_local_step", "moshpit_sgd_round", "moshpit_sgd_run", "moshpit_random_groups_round", "moshpit_random_permutation", "moshpit_refresh", "moshpit_refresh_donors", "moshpit_grouped_round", "moshpit_set_tuning", "moshpit_copy_probe", "moshpit_check_bf16_rounding", "moshpit_sync", "moshpit_last_error",
]


class MoshpitError(RuntimeError):
    pass


class _CSchedule(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("down_rounds", ctypes.c_int32), ("p", ctypes.c_double),
                ("seed", ctypes.c_uint64), ("explicit_masks", ctypes.c_void_p), ("group_skip", ctypes.c_int32),
                ("refresh", ctypes.c_int32)]


@dataclass
class Schedule:
    kind: int = SCHED_NONE
    p: float = 0.0
    seed: int = 0
    down_rounds: int = 0
    explicit_masks: np.ndarray | None = None      # uint8 [rounds, N] for SCHED_EXPLICIT
    group_skip: bool = False                      # a group with an absent member skips the round
    refresh: bool = False                         # a returning peer first copies an up-to-date peer


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libmoshpit.so (built in-tree by __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise MoshpitError(f"{LIB_PATH} is missing: run `python __graft_entry__.py` to build it")
    lib = ctypes.CDLL(LIB_PATH)
    i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    lib.moshpit_create.argtypes = [i64, i64, i32, i32, i32, ctypes.POINTER(vp)]
    lib.moshpit_destroy.argtypes = [vp]
    lib.moshpit_bind_state.argtypes = [vp, vp, i64, vp]
    lib.moshpit_round.argtypes = [vp, i64, vp]
    lib.moshpit_round_dev.argtypes = [vp, i64, vp]
    lib.moshpit_run.argtypes = [vp, i64, i32, ctypes.POINTER(_CSchedule), i32, vp, vp]
    lib.moshpit_dist_to_mean.argtypes = [vp, ctypes.POINTER(ctypes.c_double)]
    lib.moshpit_dist_to_mean_static.argtypes = [vp, i64, i64, i64, i32, vp, vp]
    lib.moshpit_dist_to_mean_subset.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_double)]
    lib.moshpit_group_keys.argtypes = [vp, i64, vp]
    lib.moshpit_schedule_mask.argtypes = [vp, ctypes.POINTER(_CSchedule), i64, i32, vp]
    lib.moshpit_dynamic_reset.argtypes = [vp]
    lib.moshpit_dynamic_round.argtypes = [vp, i64, ctypes.c_uint64, vp]
    lib.moshpit_dynamic_keys.argtypes = [vp, vp]
    lib.moshpit_local_step.argtypes = [vp, vp, vp, i64, ctypes.c_float]
    lib.moshpit_sgd_round.argtypes = [vp, i64, vp, vp, i64, ctypes.c_float]
    lib.moshpit_sgd_run.argtypes = [vp, i64, i32, ctypes.POINTER(_CSchedule), i32, vp, i64, ctypes.c_float, vp, vp]
    lib.moshpit_random_groups_round.argtypes = [vp, i64, ctypes.c_uint64, i32, vp]
    lib.moshpit_random_permutation.argtypes = [vp, i64, ctypes.c_uint64, vp]
    lib.moshpit_refresh.argtypes = [vp, i64, ctypes.c_uint64, vp, vp]
    lib.moshpit_refresh_donors.argtypes = [vp, i64, ctypes.c_uint64, vp, vp, vp]
    lib.moshpit_grouped_round.argtypes = [vp, vp, i64, i32, vp]
    lib.moshpit_set_tuning.argtypes = [vp, i32, i32, i32, i32, i32, i32]
    lib.moshpit_copy_probe.argtypes = [vp, vp, i64, vp]
    lib.moshpit_check_bf16_rounding.argtypes = [vp, vp]
    lib.moshpit_sync.argtypes = [vp]
    lib.moshpit_last_error.argtypes = [vp]
    lib.moshpit_last_error.restype = ctypes.c_char_p
    for name in EXPORTS:
        if name != "moshpit_last_error":
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _c_schedule(s: Schedule | None, rounds: int, N: int):
    if s is None:
        return None, None
    keep = None
    ptr = None
    if s.kind == SCHED_EXPLICIT:
        keep = np.ascontiguousarray(s.explicit_masks, dtype=np.uint8)
        if keep.shape != (rounds, N):
            raise ValueError("explicit masks must have shape (rounds, N)")
        ptr = keep.ctypes.data
    return _CSchedule(s.kind, s.down_rounds, float(s.p), s.seed, ptr, 1 if s.group_skip else 0, 1 if s.refresh else 0), keep


class Moshpit:
    """One handle = one peer-state matrix of N = M^d rows with P parameters."""

    def __init__(self, N: int, P: int, M: int, d: int, dtype: int):
        self._lib = load_library()
        self._h = ctypes.c_void_p()
        rc = self._lib.moshpit_create(N, P, M, d, dtype, ctypes.byref(self._h))
        if rc != 0:
            msg = self._lib.moshpit_last_error(None).decode()
            self._h = ctypes.c_void_p()
            raise MoshpitError(f"moshpit_create failed ({rc}): {msg}")
        self.N, self.P, self.M, self.d, self.dtype = N, P, M, d, dtype
        self._state = None

    # -- plumbing ---------------------------------------------------------
    def _check(self, rc: int, what: str) -> None:
        if rc != 0:
            raise MoshpitError(f"{what} failed ({rc}): {self._lib.moshpit_last_error(self._h).decode()}")

    def close(self) -> None:
        if self._h:
            self._lib.moshpit_destroy(self._h)
            self._h = ctypes.c_void_p()
            self._state = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- the C ABI, one method per entry point ------------------------------
    def bind_state(self, X, stream=None) -> None:
        """X: torch tensor [N, P] on the GPU (float32 or bfloat16), unit column stride."""
        import torch
        want = torch.float32 if self.dtype == F32 else torch.bfloat16
        if X.dtype != want or X.dim() != 2 or tuple(X.shape) != (self.N, self.P) or not X.is_cuda:
            raise ValueError("state tensor has the wrong dtype, shape or device")
        if X.stride(1) != 1:
            raise ValueError("state tensor must have unit column stride")
        if stream is None:
            stream = torch.cuda.current_stream(X.device)
        self._check(self._lib.moshpit_bind_state(self._h, X.data_ptr(), X.stride(0), stream.cuda_stream), "bind_state")
        self._state = (X, stream)              # keep both alive

    def bind_raw(self, ptr: int, row_stride: int, stream_handle: int = 0) -> None:
        self._check(self._lib.moshpit_bind_state(self._h, ptr, row_stride, stream_handle), "bind_state")

    def round(self, t: int, alive=None) -> None:
        if alive is None:
            self._check(self._lib.moshpit_round(self._h, t, None), "round")
            return
        a = np.ascontiguousarray(alive, dtype=np.uint8)
        if a.shape != (self.N,):
            raise ValueError("alive mask must have shape (N,)")
        self._check(self._lib.moshpit_round(self._h, t, a.ctypes.data), "round")

    def round_dev(self, t: int, alive_dev) -> None:
        """alive_dev: torch uint8 tensor [N] on the GPU, or None."""
        ptr = None
        if alive_dev is not None:
            if alive_dev.numel() != self.N or alive_dev.element_size() != 1 or not alive_dev.is_contiguous():
                raise ValueError("device mask must be N contiguous bytes")
            ptr = alive_dev.data_ptr()
        self._check(self._lib.moshpit_round_dev(self._h, t, ptr), "round_dev")

    def run(self, t0: int, rounds: int, schedule: Schedule | None = None, want_dist: bool = False,
            want_times: bool = False, flags: int = 0):
        cs, keep = _c_schedule(schedule, rounds, self.N)
        dist = np.zeros(rounds + 1, dtype=np.float64) if want_dist else None
        ms = np.zeros(rounds, dtype=np.float32) if want_times else None
        rc = self._lib.moshpit_run(self._h, t0, rounds, ctypes.byref(cs) if cs is not None else None, flags,
                                   dist.ctypes.data if want_dist else None, ms.ctypes.data if want_times else None)
        self._check(rc, "run")
        del keep
        return dist, ms

    def dist_to_mean(self) -> float:
        out = ctypes.c_double()
        self._check(self._lib.moshpit_dist_to_mean(self._h, ctypes.byref(out)), "dist_to_mean")
        return out.value

    def dist_to_mean_subset(self, present) -> float:
        """present: uint8 [N], non-zero = the row holds a peer (None = all rows)."""
        out = ctypes.c_double()
        ptr = None
        if present is not None:
            keep = np.ascontiguousarray(present, dtype=np.uint8)
            if keep.shape != (self.N,):
                raise ValueError("present mask must have shape (N,)")
            ptr = keep.ctypes.data
        self._check(self._lib.moshpit_dist_to_mean_subset(self._h, ptr, ctypes.byref(out)), "dist_to_mean_subset")
        return out.value

    def group_keys(self, t: int) -> np.ndarray:
        keys = np.empty(self.N, dtype=np.int32)
        self._check(self._lib.moshpit_group_keys(self._h, t, keys.ctypes.data), "group_keys")
        return keys

    def schedule_mask(self, schedule: Schedule | None, t0: int, rounds: int) -> np.ndarray:
        cs, keep = _c_schedule(schedule, rounds, self.N)
        masks = np.empty((rounds, self.N), dtype=np.uint8)
        rc = self._lib.moshpit_schedule_mask(self._h, ctypes.byref(cs) if cs is not None else None, t0, rounds,
                                             masks.ctypes.data)
        self._check(rc, "schedule_mask")
        del keep
        return masks

    def _alive_ptr(self, alive):
        if alive is None:
            return None, None
        a = np.ascontiguousarray(alive, dtype=np.uint8)
        if a.shape != (self.N,):
            raise ValueError("alive mask must have shape (N,)")
        return a, a.ctypes.data

    def dynamic_reset(self) -> None:
        self._check(self._lib.moshpit_dynamic_reset(self._h), "dynamic_reset")

    def dynamic_round(self, t: int, seed: int, alive=None) -> None:
        keep, ptr = self._alive_ptr(alive)
        self._check(self._lib.moshpit_dynamic_round(self._h, t, seed, ptr), "dynamic_round")

    def dynamic_keys(self) -> np.ndarray:
        keys = np.zeros((self.N, max(self.d - 1, 0)), dtype=np.int32)
        self._check(self._lib.moshpit_dynamic_keys(self._h, keys.ctypes.data if keys.size else None), "dynamic_keys")
        return keys

    def _grad(self, G):
        X = self._state[0]
        if G.dtype != X.dtype or tuple(G.shape) != (self.N, self.P) or G.stride(1) != 1 or not G.is_cuda:
            raise ValueError("gradient tensor must match the state's dtype, shape and device")
        return G.data_ptr(), G.stride(0)

    def local_step(self, G, gamma: float, alive=None) -> None:
        keep, ptr = self._alive_ptr(alive)
        gp, gs = self._grad(G)
        self._check(self._lib.moshpit_local_step(self._h, ptr, gp, gs, gamma), "local_step")

    def sgd_round(self, t: int, G, gamma: float, alive=None) -> None:
        keep, ptr = self._alive_ptr(alive)
        gp, gs = self._grad(G)
        self._check(self._lib.moshpit_sgd_round(self._h, t, ptr, gp, gs, gamma), "sgd_round")

    def sgd_run(self, t0: int, rounds: int, G, gamma: float, schedule: Schedule | None = None, want_dist: bool = False,
                want_times: bool = False, flags: int = 0):
        cs, keep = _c_schedule(schedule, rounds, self.N)
        gp, gs = self._grad(G)
        dist = np.zeros(rounds + 1, dtype=np.float64) if want_dist else None
        ms = np.zeros(rounds, dtype=np.float32) if want_times else None
        rc = self._lib.moshpit_sgd_run(self._h, t0, rounds, ctypes.byref(cs) if cs is not None else None, flags, gp, gs,
                                       gamma, dist.ctypes.data if want_dist else None,
                                       ms.ctypes.data if want_times else None)
        self._check(rc, "sgd_run")
        del keep
        return dist, ms

    def random_groups_round(self, t: int, seed: int, group_size: int, alive=None) -> None:
        keep, ptr = self._alive_ptr(alive)
        self._check(self._lib.moshpit_random_groups_round(self._h, t, seed, group_size, ptr), "random_groups_round")

    def random_permutation(self, t: int, seed: int) -> np.ndarray:
        perm = np.empty(self.N, dtype=np.int32)
        self._check(self._lib.moshpit_random_permutation(self._h, t, seed, perm.ctypes.data), "random_permutation")
        return perm

    def _two_masks(self, prev, cur):
        a = np.ascontiguousarray(prev, dtype=np.uint8)
        b = np.ascontiguousarray(cur, dtype=np.uint8)
        if a.shape != (self.N,) or b.shape != (self.N,):
            raise ValueError("masks must have shape (N,)")
        return a, b

    def refresh(self, t: int, seed: int, alive_prev, alive_cur) -> None:
        a, b = self._two_masks(alive_prev, alive_cur)
        self._check(self._lib.moshpit_refresh(self._h, t, seed, a.ctypes.data, b.ctypes.data), "refresh")

    def refresh_donors(self, t: int, seed: int, alive_prev, alive_cur) -> np.ndarray:
        a, b = self._two_masks(alive_prev, alive_cur)
        donors = np.empty(self.N, dtype=np.int32)
        self._check(self._lib.moshpit_refresh_donors(self._h, t, seed, a.ctypes.data, b.ctypes.data,
                                                     donors.ctypes.data), "refresh_donors")
        return donors

    def grouped_round(self, index, group_size: int, alive=None) -> None:
        idx = np.ascontiguousarray(index, dtype=np.int32)
        keep, ptr = self._alive_ptr(alive)
        self._check(self._lib.moshpit_grouped_round(self._h, idx.ctypes.data, len(idx), group_size, ptr),
                    "grouped_round")

    def set_tuning(self, cols: int = 0, unroll: int = 0, nontemporal: int = -1, block: int = 0,
                   waves_per_cu: int = 0, order: int = -1) -> None:
        self._check(self._lib.moshpit_set_tuning(self._h, cols, unroll, nontemporal, block, waves_per_cu, order),
                    "set_tuning")

    def sync(self) -> None:
        self._check(self._lib.moshpit_sync(self._h), "sync")


def copy_probe(dst, src, stream=None) -> None:
    """Queue the library's plain copy kernel dst <- src (torch GPU tensors of equal byte size)."""
    import torch
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != nbytes:
        raise ValueError("size mismatch")
    if stream is None:
        stream = torch.cuda.current_stream(src.device)
    rc = load_library().moshpit_copy_probe(dst.data_ptr(), src.data_ptr(), nbytes, stream.cuda_stream)
    if rc != 0:
        raise MoshpitError(f"copy_probe failed ({rc})")


def check_bf16_rounding(stream=None) -> int:
    """Number of binary32 inputs (of all 2^32) on which the hardware bfloat16 rounding the
    kernels use differs from its integer definition; waits for the result."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    out = ctypes.c_uint64(2**64 - 1)
    rc = load_library().moshpit_check_bf16_rounding(stream.cuda_stream, ctypes.byref(out))
    if rc != 0:
        raise MoshpitError(f"check_bf16_rounding failed ({rc})")
    return int(out.value)


def dist_to_mean_static(X, out, stream=None) -> None:
    """Queue the allocation-free distortion of the [N, P] GPU tensor X (float32 or bfloat16,
    unit column stride) into out (GPU tensor holding one float64).  Returns without waiting."""
    import torch
    if X.dim() != 2 or X.stride(1) != 1 or not X.is_cuda or X.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("state tensor has the wrong dtype, shape or device")
    if out.dtype != torch.float64 or out.numel() != 1 or not out.is_cuda:
        raise ValueError("out must be one float64 on the GPU")
    if stream is None:
        stream = torch.cuda.current_stream(X.device)
    lib = load_library()
    rc = lib.moshpit_dist_to_mean_static(X.data_ptr(), X.shape[0], X.shape[1], X.stride(0),
                                         F32 if X.dtype == torch.float32 else BF16, stream.cuda_stream, out.data_ptr())
    if rc != 0:
        raise MoshpitError(f"dist_to_mean_static failed ({rc}): {lib.moshpit_last_error(None).decode()}")
