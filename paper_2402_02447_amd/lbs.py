"""ctypes binding of the load-balancing simulation in libbca.so (include/lbs.h):
same names as the C ABI, argument marshalling only; every draw, sort and sum runs
in the library's HIP kernels.  Raises if the library is missing."""
from __future__ import annotations

import ctypes as C
from typing import Optional, Sequence

import numpy as np

from .binding import _ptr, _stream, load_library

LBS_NONE, LBS_STRATIFIED, LBS_LOCAL_RASTER, LBS_LOCAL_SNAKE, LBS_GLOBAL = 0, 1, 2, 3, 4
LBS_MAX_LEN, LBS_MAX_STRATA, LBS_MAX_LOCAL_BATCH, LBS_MAX_NODE_POOL = 1024, 8, 64, 1024
_ERR = {-1: "LBS_ERR_NULL", -2: "LBS_ERR_ARG", -3: "LBS_ERR_LIMIT", -4: "LBS_ERR_HIP", -5: "LBS_ERR_HOST"}

EXPORTS = ["lbs_dataset_create", "lbs_dataset_destroy", "lbs_simulate", "lbs_simulate_all", "lbs_issue_rate_probe",
           "lbs_last_error"]
PROBE_KINDS = {0: ("v_xor_b32 + v_add_u32", 2), 1: ("v_mul_lo_u32 (+ add)", 1), 2: ("v_mul_hi_u32 + v_add_u32", 2),
               3: ("v_med3_u32", 1), 4: ("DPP v_mov_b32 + v_add_u32", 2), 5: ("ds_bpermute_b32 + v_add_u32", 2),
               6: ("v_fma_f32", 1)}       # kind -> (instructions, how many of them per round and chain)


class LbsError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_ERR.get(code, code)}: {msg}")
        self.code = code


class _Run(C.Structure):
    _fields_ = [("method", C.c_uint32), ("local_batch", C.c_uint32), ("gpus_per_node", C.c_uint32),
                ("n_gpus", C.c_uint32), ("quota", C.c_uint32 * LBS_MAX_STRATA), ("seed", C.c_uint64),
                ("first_trial", C.c_uint64), ("n_trials", C.c_uint64)]


_declared = False


def _lib():
    global _declared
    L = load_library()
    if not _declared:
        vp, u32, u64 = C.c_void_p, C.c_uint32, C.c_uint64
        L.lbs_dataset_create.argtypes = [C.POINTER(vp), C.c_int, u32, C.POINTER(u32), u32, C.POINTER(u32)]
        L.lbs_dataset_destroy.argtypes = [vp]
        L.lbs_dataset_destroy.restype = None
        L.lbs_simulate.argtypes = [vp, C.POINTER(_Run), vp, vp, vp, vp]
        L.lbs_simulate_all.argtypes = [vp, C.POINTER(_Run), vp, vp, vp, vp]
        L.lbs_issue_rate_probe.argtypes = [C.c_int, u32, u32, vp, vp]
        L.lbs_last_error.restype = C.c_char_p
        for name in EXPORTS:
            getattr(L, name)
        _declared = True
    return L


def _check(rc: int) -> None:
    if rc != 0:
        raise LbsError(rc, _lib().lbs_last_error().decode())


def issue_rate_probe(kind: int, n_workgroups: int, iters: int, out, stream=None) -> None:
    """lbs_issue_rate_probe: enqueue the register-arithmetic probe of one instruction kind (measurement only)."""
    _check(_lib().lbs_issue_rate_probe(kind, n_workgroups, iters, _ptr(out), _stream(stream)))


class Dataset:
    """A length histogram with its strata on one device (lbs_dataset_create / destroy)."""

    def __init__(self, cum: Sequence[int], stratum_end: Sequence[int], device: int = 0):
        L = _lib()
        self._L = L
        self._h = C.c_void_p()
        c = np.ascontiguousarray(cum, dtype=np.uint32)
        se = np.ascontiguousarray(stratum_end, dtype=np.uint32)
        u32p = C.POINTER(C.c_uint32)
        _check(L.lbs_dataset_create(C.byref(self._h), device, len(c) - 1, c.ctypes.data_as(u32p), len(se),
                                    se.ctypes.data_as(u32p)))
        self.n_strata = len(se)

    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._L.lbs_dataset_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def lbs_simulate(self, method: int, local_batch: int, gpus_per_node: int, n_gpus: int, quota: Optional[Sequence[int]],
                     seed: int, n_trials: int, sums, trial_min=None, trial_max=None, first_trial: int = 0,
                     stream=None) -> None:
        """sums: device buffer of two uint64; trial_min / trial_max: device buffers of n_trials uint32 or None."""
        run = _Run(method, local_batch, gpus_per_node, n_gpus, (C.c_uint32 * LBS_MAX_STRATA)(), seed, first_trial,
                   n_trials)
        if quota is not None:
            if len(quota) > LBS_MAX_STRATA:
                raise ValueError("too many strata")
            for i, q in enumerate(quota):
                run.quota[i] = int(q)
        _check(self._L.lbs_simulate(self._h, C.byref(run), _ptr(trial_min), _ptr(trial_max), _ptr(sums), _stream(stream)))

    def lbs_simulate_all(self, local_batch: int, gpus_per_node: int, n_gpus: int, quota: Sequence[int], seed: int,
                         n_trials: int, sums, trial_min=None, trial_max=None, first_trial: int = 0, stream=None) -> None:
        """All five methods on the same draws.  sums: device buffer of 5 x 2 uint64; trial_min / trial_max: device
        buffers of 5 x n_trials uint32 or None."""
        run = _Run(0, local_batch, gpus_per_node, n_gpus, (C.c_uint32 * LBS_MAX_STRATA)(), seed, first_trial, n_trials)
        if len(quota) > LBS_MAX_STRATA:
            raise ValueError("too many strata")
        for i, q in enumerate(quota):
            run.quota[i] = int(q)
        _check(self._L.lbs_simulate_all(self._h, C.byref(run), _ptr(trial_min), _ptr(trial_max), _ptr(sums), _stream(stream)))
