"""ctypes front end of the load-balancing simulation oracle (oracle/lbs_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg; never by the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

NONE, STRATIFIED, LOCAL_RASTER, LOCAL_SNAKE, GLOBAL = 0, 1, 2, 3, 4

_lib = None


def lib(path: Optional[str] = None):
    global _lib
    if path is not None:
        return _declare(C.CDLL(path))
    if _lib is None:
        so = os.environ.get("LBS_ORACLE_LIB") or (_build.LBS_LIB if os.path.exists(_build.LBS_LIB) else _build.build_lbs())
        _lib = _declare(C.CDLL(so))
    return _lib


def _declare(L):
    u32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)
    L.orc_lbs_splitmix64.argtypes = [C.c_uint64, C.c_uint64]
    L.orc_lbs_splitmix64.restype = C.c_uint64
    L.orc_lbs_length_of.argtypes = [u32p, C.c_uint32, C.c_uint32]
    L.orc_lbs_length_of.restype = C.c_uint32
    L.orc_lbs_draw.argtypes = [u32p, C.c_uint32, C.c_int, C.c_uint32, u32p, u32p, C.c_uint32, C.c_uint32, C.c_uint64,
                               C.c_uint64, C.c_uint32, u32p]
    L.orc_lbs_draw.restype = None
    L.orc_lbs_presort_scatter.argtypes = [u32p, C.c_uint32, C.c_uint32, C.c_int, u64p]
    L.orc_lbs_presort_scatter.restype = None
    L.orc_lbs_simulate.argtypes = [u32p, C.c_uint32, C.c_uint32, u32p, u32p, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int,
                                   C.c_uint64, C.c_uint64, C.c_uint64, u32p, u32p, u64p]
    L.orc_lbs_simulate.restype = C.c_int
    return L


def _u32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.uint32)


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


def splitmix64(seed: int, k: int) -> int:
    return int(lib().orc_lbs_splitmix64(seed, k))


def length_of(cum: Sequence[int], index: int) -> int:
    c = _u32(cum)
    return int(lib().orc_lbs_length_of(_p(c), len(c) - 1, index))


def draw(cum, stratified: bool, stratum_end, quota, local_batch: int, n_gpus: int, seed: int, trial: int,
         gpu: int) -> np.ndarray:
    c, se, q = _u32(cum), _u32(stratum_end), _u32(quota)
    out = np.zeros(local_batch, np.uint32)
    lib().orc_lbs_draw(_p(c), len(c) - 1, int(stratified), len(se), _p(se), _p(q), local_batch, n_gpus, seed, trial, gpu,
                       _p(out))
    return out


def presort_scatter(lengths, n_group: int, local_batch: int, snake: bool) -> np.ndarray:
    """Token count per GPU after sorting the group's sequences and dealing them row by row."""
    a = _u32(lengths).copy()
    assert a.shape[0] == n_group * local_batch
    tokens = np.zeros(n_group, np.uint64)
    lib().orc_lbs_presort_scatter(_p(a), n_group, local_batch, int(snake), tokens.ctypes.data_as(C.POINTER(C.c_uint64)))
    return tokens


def simulate(cum, stratum_end, quota, local_batch: int, gpus_per_node: int, n_gpus: int, method: int, seed: int,
             n_trials: int, first_trial: int = 0) -> Tuple[np.ndarray, np.ndarray, int, int]:
    """Returns (per-trial min, per-trial max, sum of mins, sum of maxes)."""
    c, se, q = _u32(cum), _u32(stratum_end), _u32(quota)
    tmin = np.zeros(max(1, n_trials), np.uint32)
    tmax = np.zeros(max(1, n_trials), np.uint32)
    sums = np.zeros(2, np.uint64)
    rc = lib().orc_lbs_simulate(_p(c), len(c) - 1, len(se), _p(se), _p(q), local_batch, gpus_per_node, n_gpus, method,
                                seed, first_trial, n_trials, _p(tmin), _p(tmax),
                                sums.ctypes.data_as(C.POINTER(C.c_uint64)))
    if rc != 0:
        raise ValueError("orc_lbs_simulate: arguments outside the definition")
    return tmin[:n_trials], tmax[:n_trials], int(sums[0]), int(sums[1])
