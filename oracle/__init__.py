"""ctypes front end of the CPU oracle (oracle/bca_oracle.cpp).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  It does not import the GPU package and the GPU
package does not import it.

All functions take plain numpy arrays.  A "tensor list" is a Python list of 1-D
numpy arrays, one per tensor (float32 or float16 gradients, or bfloat16 gradients
wrapped in `Bf16`; float64 state).
Layout arguments are the five arrays of a bucket layout: tensor_numel,
bucket_seg_off, seg_tensor, seg_begin, seg_len.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

STATUS_NONFINITE = 1
STATUS_BAD_THRESHOLD = 2

_lib = None


def lib(path: Optional[str] = None):
    """Load (building first if no library is there) the oracle shared object."""
    global _lib
    if path is not None:
        return _declare(C.CDLL(path))
    if _lib is None:
        # BCA_ORACLE_LIB lets the mutation test point the pin tests at a deliberately broken build
        so = os.environ.get("BCA_ORACLE_LIB") or (_build.LIB if os.path.exists(_build.LIB) else _build.build())
        _lib = _declare(C.CDLL(so))
    return _lib


def _declare(L):
    u32p, u64p = C.POINTER(C.c_uint32), C.POINTER(C.c_uint64)
    vpp = C.POINTER(C.c_void_p)
    dp, fp = C.POINTER(C.c_double), C.POINTER(C.c_float)
    L.orc_half_to_double.argtypes = [C.c_uint16]
    L.orc_half_to_double.restype = C.c_double
    L.orc_float_to_half.argtypes = [C.c_float]
    L.orc_float_to_half.restype = C.c_uint16
    L.orc_bf16_to_double.argtypes = [C.c_uint16]
    L.orc_bf16_to_double.restype = C.c_double
    L.orc_float_to_bf16.argtypes = [C.c_float]
    L.orc_float_to_bf16.restype = C.c_uint16
    L.orc_alg1_threshold.argtypes = [C.c_double, C.c_uint64]
    L.orc_alg1_threshold.restype = C.c_double
    L.orc_bucket_norms.argtypes = [C.c_uint32, u64p, u32p, u64p, u64p, vpp, C.c_int, dp]
    L.orc_bucket_norms.restype = None
    L.orc_clip_coefs.argtypes = [C.c_uint32, dp, fp, fp]
    L.orc_clip_coefs.restype = C.c_int32
    L.orc_bucket_scale.argtypes = [C.c_uint32, u64p, u32p, u64p, u64p, vpp, C.c_int, fp]
    L.orc_bucket_scale.restype = None
    u8p = C.POINTER(C.c_uint8)
    L.orc_adam_step.argtypes = [C.c_uint32, u64p, vpp, C.c_int, vpp, vpp, vpp,
                                C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint64, u8p]
    L.orc_adam_step.restype = None
    L.orc_bucket_clip_adam.argtypes = [C.c_uint32, u64p, u32p, u64p, u64p, vpp, C.c_int, vpp, vpp, vpp, fp,
                                       C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint64,
                                       C.c_int, C.c_int, dp, fp, u8p]
    L.orc_bucket_clip_adam.restype = C.c_int32
    L.orc_whole_clip_adam.argtypes = [C.c_uint32, u64p, u32p, u64p, u64p, vpp, C.c_int, vpp, vpp, vpp, C.c_float,
                                      C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint64, C.c_int,
                                      dp, dp, fp, u8p]
    L.orc_whole_clip_adam.restype = C.c_int32
    L.orc_lamb_step.argtypes = [C.c_uint32, u64p, vpp, C.c_int, vpp, vpp, vpp,
                                C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint64, u8p, dp]
    L.orc_lamb_step.restype = None
    L.orc_bucket_clip_lamb.argtypes = [C.c_uint32, u64p, C.c_uint32, u64p, u32p, u64p, u64p, vpp, C.c_int, vpp, vpp, vpp,
                                       fp, C.c_double, C.c_double, C.c_double, C.c_double, C.c_double, C.c_uint64,
                                       C.c_int, u8p, dp, fp, dp]
    L.orc_bucket_clip_lamb.restype = C.c_int32
    L.orc_compare_f32.argtypes = [fp, dp, C.c_uint64, C.c_double, C.c_double, C.c_double, C.c_double, dp]
    L.orc_compare_f32.restype = C.c_uint64
    return L


# ---------------------------------------------------------------- marshalling


def _p(a: np.ndarray, ty):
    return a.ctypes.data_as(C.POINTER(ty))


def _ptr_array(tensors: Sequence[np.ndarray], dtype) -> "C.Array":
    arr = (C.c_void_p * max(1, len(tensors)))()
    for i, t in enumerate(tensors):
        if t.dtype != dtype or not t.flags["C_CONTIGUOUS"] or t.ndim != 1:
            raise TypeError(f"tensor {i}: need 1-D contiguous {dtype}, got {t.dtype} {t.shape}")
        arr[i] = t.ctypes.data
    return arr


class Bf16(list):
    """A tensor list of bfloat16 gradients: 1-D uint16 arrays holding the bit patterns
    (numpy has no bfloat16 type)."""


def _gdt(grads: Sequence[np.ndarray]) -> Tuple[int, type]:
    if isinstance(grads, Bf16):
        return 2, np.uint16
    if len(grads) == 0:
        return 0, np.float32
    dt = grads[0].dtype
    if dt == np.float32:
        return 0, np.float32
    if dt == np.float16:
        return 1, np.float16
    raise TypeError(f"gradient dtype {dt} not supported")


def _mask(decay, n_tensors: int):
    """Per-tensor weight-decay mask as (keep-alive array, pointer); None means decay everywhere."""
    if decay is None:
        return None, None
    a = np.ascontiguousarray(decay, dtype=np.uint8)
    assert a.shape == (n_tensors,)
    if n_tensors == 0:
        a = np.zeros(1, np.uint8)
    return a, _p(a, C.c_uint8)


class _Lay:
    def __init__(self, layout):
        self.numel = np.ascontiguousarray(layout.tensor_numel, dtype=np.uint64)
        self.off = np.ascontiguousarray(layout.bucket_seg_off, dtype=np.uint64)
        self.st = np.ascontiguousarray(layout.seg_tensor, dtype=np.uint32)
        self.sb = np.ascontiguousarray(layout.seg_begin, dtype=np.uint64)
        self.sl = np.ascontiguousarray(layout.seg_len, dtype=np.uint64)
        self.nb = int(self.off.shape[0]) - 1
        self.nt = int(self.numel.shape[0])
        # keep one spare entry so that empty arrays still have a valid address
        if self.st.shape[0] == 0:
            self.st = np.zeros(1, np.uint32)
            self.sb = np.zeros(1, np.uint64)
            self.sl = np.zeros(1, np.uint64)

    def args(self):
        return (C.c_uint32(self.nb), _p(self.off, C.c_uint64), _p(self.st, C.c_uint32),
                _p(self.sb, C.c_uint64), _p(self.sl, C.c_uint64))


# ---------------------------------------------------------------- public API


def half_to_double(bits: int) -> float:
    return float(lib().orc_half_to_double(int(bits)))


def float_to_half(x: float) -> int:
    return int(lib().orc_float_to_half(C.c_float(x)))


def bf16_to_double(bits: int) -> float:
    return float(lib().orc_bf16_to_double(int(bits)))


def float_to_bf16(x: float) -> int:
    return int(lib().orc_float_to_bf16(C.c_float(x)))


def alg1_threshold(c: float, n_buckets: int) -> float:
    """Per-bucket threshold of Alg. 1: c / sqrt(B)."""
    return float(lib().orc_alg1_threshold(float(c), int(n_buckets)))


def bucket_norms(layout, grads: Sequence[np.ndarray]) -> np.ndarray:
    la = _Lay(layout)
    gdt, dt = _gdt(grads)
    norms = np.zeros(max(1, la.nb), np.float64)
    lib().orc_bucket_norms(*la.args(), _ptr_array(grads, dt), gdt, _p(norms, C.c_double))
    return norms[:la.nb]


def clip_coefs(norms: np.ndarray, thresholds: np.ndarray) -> Tuple[np.ndarray, int]:
    norms = np.ascontiguousarray(norms, np.float64)
    thr = np.ascontiguousarray(thresholds, np.float32)
    assert norms.shape == thr.shape
    nb = norms.shape[0]
    coefs = np.ones(max(1, nb), np.float32)
    st = lib().orc_clip_coefs(nb, _p(norms, C.c_double), _p(thr, C.c_float), _p(coefs, C.c_float))
    return coefs[:nb], int(st)


def bucket_scale(layout, grads: List[np.ndarray], coefs: np.ndarray) -> None:
    """grads are scaled in place, in their own storage type."""
    la = _Lay(layout)
    gdt, dt = _gdt(grads)
    cf = np.ascontiguousarray(coefs, np.float32)
    assert cf.shape[0] == la.nb
    lib().orc_bucket_scale(*la.args(), _ptr_array(grads, dt), gdt, _p(cf, C.c_float))


def adam_step(layout_or_numel, grads: Sequence[np.ndarray], p: List[np.ndarray], m: List[np.ndarray],
              v: List[np.ndarray], lr: float, beta1: float, beta2: float, eps: float, weight_decay: float,
              step: int, decay=None) -> None:
    """p, m, v (float64) are updated in place from the stored gradients.  decay: optional
    per-tensor mask (non-zero = weight decay applies to that tensor)."""
    numel = getattr(layout_or_numel, "tensor_numel", layout_or_numel)
    numel = np.ascontiguousarray(numel, np.uint64)
    gdt, dt = _gdt(grads)
    for t, n in enumerate(numel):
        assert grads[t].shape[0] == p[t].shape[0] == m[t].shape[0] == v[t].shape[0] == int(n)
    keep, dm = _mask(decay, numel.shape[0])
    lib().orc_adam_step(numel.shape[0], _p(numel, C.c_uint64), _ptr_array(grads, dt), gdt,
                        _ptr_array(p, np.float64), _ptr_array(m, np.float64), _ptr_array(v, np.float64),
                        lr, beta1, beta2, eps, weight_decay, int(step), dm)


def lamb_step(layout_or_numel, grads: Sequence[np.ndarray], p: List[np.ndarray], m: List[np.ndarray],
              v: List[np.ndarray], lr: float, beta1: float, beta2: float, eps: float, weight_decay: float,
              step: int, decay=None) -> np.ndarray:
    """LAMB on the stored gradients; p, m, v (float64) updated in place.  Returns the per-tensor trust ratios."""
    numel = getattr(layout_or_numel, "tensor_numel", layout_or_numel)
    numel = np.ascontiguousarray(numel, np.uint64)
    gdt, dt = _gdt(grads)
    for t, n in enumerate(numel):
        assert grads[t].shape[0] == p[t].shape[0] == m[t].shape[0] == v[t].shape[0] == int(n)
    keep, dm = _mask(decay, numel.shape[0])
    trust = np.ones(max(1, numel.shape[0]), np.float64)
    lib().orc_lamb_step(numel.shape[0], _p(numel, C.c_uint64), _ptr_array(grads, dt), gdt,
                        _ptr_array(p, np.float64), _ptr_array(m, np.float64), _ptr_array(v, np.float64),
                        lr, beta1, beta2, eps, weight_decay, int(step), dm, _p(trust, C.c_double))
    return trust[:numel.shape[0]]


def bucket_clip_lamb(layout, grads: List[np.ndarray], p: List[np.ndarray], m: List[np.ndarray],
                     v: List[np.ndarray], thresholds: np.ndarray, lr: float, beta1: float, beta2: float,
                     eps: float, weight_decay: float, step: int, write_back: bool = False, decay=None):
    """Bucket-wise clipping, then LAMB.  Returns (norms float64, coefs float32, trust float64, status bits)."""
    la = _Lay(layout)
    gdt, dt = _gdt(grads)
    thr = np.ascontiguousarray(thresholds, np.float32)
    assert thr.shape[0] == la.nb
    for t in range(la.nt):
        assert grads[t].shape[0] == p[t].shape[0] == m[t].shape[0] == v[t].shape[0] == int(la.numel[t])
    norms = np.zeros(max(1, la.nb), np.float64)
    coefs = np.ones(max(1, la.nb), np.float32)
    trust = np.ones(max(1, la.nt), np.float64)
    keep, dm = _mask(decay, la.nt)
    st = lib().orc_bucket_clip_lamb(C.c_uint32(la.nt), _p(la.numel, C.c_uint64), *la.args(), _ptr_array(grads, dt), gdt,
                                    _ptr_array(p, np.float64), _ptr_array(m, np.float64), _ptr_array(v, np.float64),
                                    _p(thr, C.c_float), lr, beta1, beta2, eps, weight_decay, int(step),
                                    int(write_back), dm, _p(norms, C.c_double), _p(coefs, C.c_float),
                                    _p(trust, C.c_double))
    return norms[:la.nb], coefs[:la.nb], trust[:la.nt], int(st)


def bucket_clip_adam(layout, grads: List[np.ndarray], p: List[np.ndarray], m: List[np.ndarray],
                     v: List[np.ndarray], thresholds: np.ndarray, lr: float, beta1: float, beta2: float,
                     eps: float, weight_decay: float, step: int, write_back: bool = False,
                     skip_on_nonfinite: bool = False, decay=None) -> Tuple[np.ndarray, np.ndarray, int]:
    """Fused step.  Returns (norms float64, coefs float32, status bits)."""
    la = _Lay(layout)
    gdt, dt = _gdt(grads)
    thr = np.ascontiguousarray(thresholds, np.float32)
    assert thr.shape[0] == la.nb
    for t in range(la.nt):
        assert grads[t].shape[0] == p[t].shape[0] == m[t].shape[0] == v[t].shape[0] == int(la.numel[t])
    norms = np.zeros(max(1, la.nb), np.float64)
    coefs = np.ones(max(1, la.nb), np.float32)
    keep, dm = _mask(decay, la.nt)
    st = lib().orc_bucket_clip_adam(*la.args(), _ptr_array(grads, dt), gdt, _ptr_array(p, np.float64),
                                    _ptr_array(m, np.float64), _ptr_array(v, np.float64), _p(thr, C.c_float),
                                    lr, beta1, beta2, eps, weight_decay, int(step), int(write_back),
                                    int(skip_on_nonfinite), _p(norms, C.c_double), _p(coefs, C.c_float), dm)
    return norms[:la.nb], coefs[:la.nb], int(st)


def whole_clip_adam(layout, grads: List[np.ndarray], p: List[np.ndarray], m: List[np.ndarray], v: List[np.ndarray],
                    threshold: float, lr: float, beta1: float, beta2: float, eps: float, weight_decay: float,
                    step: int, write_back: bool = False, decay=None) -> Tuple[np.ndarray, float, float, int]:
    """Whole-gradient clipping + Adam.  Returns (per-bucket norms, whole norm, coefficient, status bits)."""
    la = _Lay(layout)
    gdt, dt = _gdt(grads)
    for t in range(la.nt):
        assert grads[t].shape[0] == p[t].shape[0] == m[t].shape[0] == v[t].shape[0] == int(la.numel[t])
    norms = np.zeros(max(1, la.nb), np.float64)
    whole = np.zeros(1, np.float64)
    coef = np.ones(1, np.float32)
    keep, dm = _mask(decay, la.nt)
    st = lib().orc_whole_clip_adam(*la.args(), _ptr_array(grads, dt), gdt, _ptr_array(p, np.float64),
                                   _ptr_array(m, np.float64), _ptr_array(v, np.float64),
                                   C.c_float(float(np.float32(threshold))), lr, beta1, beta2, eps, weight_decay,
                                   int(step), int(write_back), _p(norms, C.c_double), _p(whole, C.c_double),
                                   _p(coef, C.c_float), dm)
    return norms[:la.nb], float(whole[0]), float(coef[0]), int(st)


def compare_f32(got: np.ndarray, want: np.ndarray, rel_tol: float = 1e-5, abs_tol: float = 1e-7,
                small: float = 1e-2, tiny: float = 1e-30) -> dict:
    """Apply the acceptance rule to one array: pass where rel <= rel_tol, or
    abs <= abs_tol where |want| < small."""
    got = np.ascontiguousarray(got, np.float32)
    want = np.ascontiguousarray(want, np.float64)
    assert got.shape == want.shape
    out = np.zeros(4, np.float64)
    bad = lib().orc_compare_f32(_p(got, C.c_float), _p(want, C.c_double), got.size, rel_tol, abs_tol, small,
                                tiny, _p(out, C.c_double))
    return {"n_bad": int(bad), "max_rel_big": float(out[0]), "max_abs_small": float(out[1]),
            "max_rel_all": float(out[2]), "worst_index": int(out[3])}
