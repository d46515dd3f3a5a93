"""ctypes binding of libbca.so: same names as the C ABI, argument marshalling only.

Device buffers are passed as anything with a ``data_ptr()`` method (torch
tensors) or as plain integers; streams as a ``torch.cuda.Stream``, an integer
handle, or None for the default stream.  There is no CPU fallback: if the
shared library is missing or fails to load, importing a symbol raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

BCA_GRAD_F32, BCA_GRAD_F16, BCA_GRAD_BF16 = 0, 1, 2
BCA_STATUS_NONFINITE, BCA_STATUS_BAD_THRESHOLD = 1, 2
BCA_WRITE_BACK_GRADS, BCA_SKIP_STEP_ON_NONFINITE, BCA_CLIP_WHOLE_GRADIENT = 1, 2, 4
BCA_TUNE_MULTI_LAUNCH, BCA_TUNE_STAGE_TABLE_LDS, BCA_TUNE_TICKETS = 1, 2, 4
BCA_STATUS_TIMEOUT, BCA_STATUS_INCOMPLETE = 4, 8
BCA_TABLE_NORM, BCA_TABLE_APPLY, BCA_TABLE_LAMB = 0, 1, 2

_ERR_NAMES = {-1: "BCA_ERR_NULL", -2: "BCA_ERR_LAYOUT", -3: "BCA_ERR_RANGE", -4: "BCA_ERR_HPARAM",
              -5: "BCA_ERR_UNBOUND", -6: "BCA_ERR_HIP", -7: "BCA_ERR_DTYPE", -8: "BCA_ERR_ALIGN", -9: "BCA_ERR_NOMEM"}

EXPORTS = ["bca_alg1_thresholds", "bucket_clip_flat", "bca_plan_create", "bca_plan_bind", "bca_plan_set_decay_mask", "bca_plan_set_device_hyper", "bca_plan_destroy", "bca_plan_num_buckets",
           "bca_plan_num_groups", "bca_plan_norm_item_chunks", "bca_plan_num_work_items", "bca_plan_work_item", "bca_plan_num_lamb_runs", "bca_plan_lamb_run", "bca_plan_num_chunks", "bca_plan_chunk_info", "bca_plan_bucket_chunks",
           "bucket_clip_norms", "bucket_clip_apply", "bucket_clip", "adam_step", "bucket_clip_adam", "lamb_step",
           "bucket_clip_lamb", "bca_plan_profile", "bca_plan_profile_read", "bca_plan_wait_stats", "bca_copy_bytes", "bca_last_error",
           "bca_version"]


class BcaError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


class _Segment(C.Structure):
    _fields_ = [("tensor", C.c_uint32), ("reserved", C.c_uint32), ("begin", C.c_uint64), ("len", C.c_uint64)]


class _Adam(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double)]


class _Tuning(C.Structure):
    _fields_ = [("chunk_norm", C.c_uint32), ("chunk_apply", C.c_uint32), ("grid_norm", C.c_uint32),
                ("grid_apply", C.c_uint32), ("unroll_apply", C.c_uint32), ("flags", C.c_uint32),
                ("group_bytes", C.c_uint64), ("adam_lds_reserve", C.c_uint32), ("spin_limit", C.c_uint32),
                ("norm_item_chunks", C.c_uint32), ("norm_lead", C.c_uint32), ("lamb_group_elems", C.c_uint64)]


@dataclass
class AdamHyper:
    lr: float = 1e-3
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-6
    weight_decay: float = 0.01

    def _c(self) -> _Adam:
        return _Adam(self.lr, self.beta1, self.beta2, self.eps, self.weight_decay)


def _hp(hp: Optional[AdamHyper]):
    """byref of the C struct, or NULL (allowed once the plan takes hyper-parameters from device memory)."""
    return C.byref(hp._c()) if hp is not None else None


def pack_device_hyper(hp: Optional[AdamHyper], step: int) -> bytes:
    """The 48 bytes of a bca_adam_device: copy them into a device buffer and hand that to Plan.set_device_hyper."""
    import struct
    return struct.pack("<5dQ", hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, step)


def library_path() -> str:
    return os.environ.get("BCA_LIB") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libbca.so")


_lib = None


def load_library():
    """Load libbca.so.  Raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is not None:
        return _lib
    # A process must hold one HIP runtime only.  PyTorch-ROCm ships its own
    # libamdhip64 (same soname as the system one); importing torch first makes the
    # loader resolve libbca's dependency to that copy, so that device pointers and
    # streams created by torch are valid in libbca's calls.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} not found: build it first (python -c 'import __graft_entry__ as g; g.build()')")
    L = C.CDLL(path)
    vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
    L.bca_plan_create.argtypes = [C.POINTER(vp), i32, u32, C.POINTER(u64), u32, C.POINTER(u64), C.POINTER(_Segment), i32,
                                  C.POINTER(_Tuning)]
    L.bca_plan_bind.argtypes = [vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp)]
    L.bca_plan_set_decay_mask.argtypes = [vp, C.POINTER(C.c_uint8)]
    L.bca_plan_set_device_hyper.argtypes = [vp, vp]
    L.bca_plan_destroy.argtypes = [vp]
    L.bca_plan_destroy.restype = None
    L.bca_plan_num_buckets.argtypes = [vp]
    L.bca_plan_num_buckets.restype = u32
    L.bca_plan_num_groups.argtypes = [vp]
    L.bca_plan_num_groups.restype = u32
    L.bca_plan_norm_item_chunks.argtypes = [vp]
    L.bca_plan_norm_item_chunks.restype = u32
    L.bca_plan_num_work_items.argtypes = [vp]
    L.bca_plan_num_work_items.restype = u32
    L.bca_plan_work_item.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(u32), C.POINTER(u32)]
    L.bca_plan_num_lamb_runs.argtypes = [vp]
    L.bca_plan_num_lamb_runs.restype = u32
    L.bca_plan_lamb_run.argtypes = [vp, u32, C.POINTER(u32), C.POINTER(u32)]
    L.bca_plan_num_chunks.argtypes = [vp, i32]
    L.bca_plan_num_chunks.restype = u32
    L.bca_plan_chunk_info.argtypes = [vp, i32, u32, C.POINTER(u32), C.POINTER(u64), C.POINTER(u32), C.POINTER(u32)]
    L.bca_plan_bucket_chunks.argtypes = [vp, i32, u32, C.POINTER(u32), C.POINTER(u32)]
    L.bucket_clip_norms.argtypes = [vp, u32, u32, vp, vp]
    L.bucket_clip_apply.argtypes = [vp, u32, u32, vp, vp, vp, vp, vp]
    L.bucket_clip.argtypes = [vp, u32, u32, vp, vp, vp, vp, vp]
    L.adam_step.argtypes = [vp, C.POINTER(_Adam), u64, vp]
    L.bucket_clip_adam.argtypes = [vp, vp, C.POINTER(_Adam), u64, u32, vp, vp, vp, vp]
    L.lamb_step.argtypes = [vp, C.POINTER(_Adam), u64, vp, vp]
    L.bucket_clip_lamb.argtypes = [vp, vp, C.POINTER(_Adam), u64, u32, vp, vp, vp, vp, vp]
    L.bca_plan_profile.argtypes = [vp, u32]
    L.bca_plan_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(u32)]
    L.bca_copy_bytes.argtypes = [vp, vp, u64, vp]
    L.bca_plan_wait_stats.argtypes = [vp, C.POINTER(u64)]
    L.bca_alg1_thresholds.argtypes = [C.c_double, u32, C.POINTER(C.c_float)]
    L.bucket_clip_flat.argtypes = [vp, u64, i32, vp, vp, vp, vp, vp]
    L.bca_last_error.restype = C.c_char_p
    L.bca_version.restype = i32
    for name in EXPORTS:
        getattr(L, name)          # raises AttributeError if a declared symbol is missing
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != 0:
        raise BcaError(rc, load_library().bca_last_error().decode())


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr()) or None
    return int(x) or None


def _stream(s) -> Optional[int]:
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return int(s.cuda_stream) or None
    return int(s) or None


def copy_bytes(dst, src, nbytes: int, stream=None) -> None:
    """Plain device copy with exactly known traffic (counter calibration)."""
    _check(load_library().bca_copy_bytes(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


def alg1_thresholds(c: float, n_buckets: int) -> np.ndarray:
    """bca_alg1_thresholds: the per-bucket thresholds of Alg. 1 as a host float32 array (the library evaluates them)."""
    out = np.zeros(n_buckets, dtype=np.float32)
    _check(load_library().bca_alg1_thresholds(float(c), int(n_buckets), out.ctypes.data_as(C.POINTER(C.c_float))))
    return out


def bucket_clip_flat(g, n: int, grad_dtype: int, threshold, norm=None, coef=None, status=None, stream=None) -> None:
    """bucket_clip_flat: clip one contiguous bucket in place; no plan, no allocation (see bca.h)."""
    _check(load_library().bucket_clip_flat(_ptr(g), int(n), grad_dtype, _ptr(threshold), _ptr(norm), _ptr(coef),
                                           _ptr(status), _stream(stream)))


class Plan:
    """A bucket layout on one device (bca_plan_create / bind / destroy) and the four compute calls."""

    def __init__(self, tensor_numel: Sequence[int], bucket_seg_off: Sequence[int], seg_tensor: Sequence[int],
                 seg_begin: Sequence[int], seg_len: Sequence[int], grad_dtype: int = BCA_GRAD_F32, device: int = 0,
                 chunk_norm: int = 0, chunk_apply: int = 0, grid_norm: int = 0, grid_apply: int = 0,
                 unroll_apply: int = 0, tune_flags: int = 0, group_bytes: int = 0, adam_lds_reserve: int = 0,
                 spin_limit: int = 0, norm_item_chunks: int = 0, norm_lead: int = 0, lamb_group_elems: int = 0):
        L = load_library()
        self._L = L
        self._h = C.c_void_p()
        numel = np.ascontiguousarray(tensor_numel, dtype=np.uint64)
        off = np.ascontiguousarray(bucket_seg_off, dtype=np.uint64)
        n_seg = len(seg_tensor)
        segs = (_Segment * max(1, n_seg))()
        for i in range(n_seg):
            segs[i] = _Segment(int(seg_tensor[i]), 0, int(seg_begin[i]), int(seg_len[i]))
        tune = _Tuning(chunk_norm, chunk_apply, grid_norm, grid_apply, unroll_apply, tune_flags, group_bytes,
                       adam_lds_reserve, spin_limit, norm_item_chunks, norm_lead, lamb_group_elems)
        _check(L.bca_plan_create(C.byref(self._h), device, len(numel), numel.ctypes.data_as(C.POINTER(C.c_uint64)),
                                 len(off) - 1, off.ctypes.data_as(C.POINTER(C.c_uint64)), segs, grad_dtype,
                                 C.byref(tune)))
        self.n_tensors = len(numel)
        self.device = device
        self.grad_dtype = grad_dtype
        self._keep = None

    @classmethod
    def from_layout(cls, layout, grad_dtype: int = BCA_GRAD_F32, device: int = 0, **tuning) -> "Plan":
        """`layout` is any object with tensor_numel, bucket_seg_off, seg_tensor, seg_begin, seg_len."""
        return cls(layout.tensor_numel, layout.bucket_seg_off, layout.seg_tensor, layout.seg_begin, layout.seg_len,
                   grad_dtype, device, **tuning)

    # -- lifetime
    def close(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value:
            self._L.bca_plan_destroy(self._h)
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

    # -- introspection
    @property
    def n_buckets(self) -> int:
        return int(self._L.bca_plan_num_buckets(self._h))

    @property
    def n_groups(self) -> int:
        return int(self._L.bca_plan_num_groups(self._h))

    @property
    def norm_item_chunks(self) -> int:
        return int(self._L.bca_plan_norm_item_chunks(self._h))

    def lamb_runs(self):
        """The runs of tensors lamb_step sweeps one after the other, as (first_tensor, end_tensor) pairs."""
        a, b = C.c_uint32(), C.c_uint32()
        out = []
        for i in range(int(self._L.bca_plan_num_lamb_runs(self._h))):
            _check(self._L.bca_plan_lamb_run(self._h, i, C.byref(a), C.byref(b)))
            out.append((a.value, b.value))
        return out

    def work_items(self):
        """The fused step's work list as (kind, first, count) triples (bca_plan_work_item)."""
        k, f, c = C.c_uint32(), C.c_uint32(), C.c_uint32()
        out = []
        for i in range(int(self._L.bca_plan_num_work_items(self._h))):
            _check(self._L.bca_plan_work_item(self._h, i, C.byref(k), C.byref(f), C.byref(c)))
            out.append((k.value, f.value, c.value))
        return out

    def n_chunks(self, table: int = BCA_TABLE_APPLY) -> int:
        return int(self._L.bca_plan_num_chunks(self._h, table))

    def chunk_info(self, i: int, table: int = BCA_TABLE_APPLY):
        t, b, ln, bk = C.c_uint32(), C.c_uint64(), C.c_uint32(), C.c_uint32()
        _check(self._L.bca_plan_chunk_info(self._h, table, i, C.byref(t), C.byref(b), C.byref(ln), C.byref(bk)))
        return t.value, b.value, ln.value, bk.value

    def bucket_chunks(self, b: int, table: int = BCA_TABLE_APPLY):
        f, n = C.c_uint32(), C.c_uint32()
        _check(self._L.bca_plan_bucket_chunks(self._h, table, b, C.byref(f), C.byref(n)))
        return f.value, n.value

    # -- binding
    def bind(self, grads, params, exp_avg, exp_avg_sq) -> None:
        def arr(xs):
            if len(xs) != self.n_tensors:
                raise ValueError(f"expected {self.n_tensors} tensors, got {len(xs)}")
            a = (C.c_void_p * max(1, len(xs)))()
            for i, x in enumerate(xs):
                a[i] = _ptr(x)
            return a
        _check(self._L.bca_plan_bind(self._h, arr(grads), arr(params), arr(exp_avg), arr(exp_avg_sq)))
        self._keep = (grads, params, exp_avg, exp_avg_sq)     # keep the tensors alive while bound

    def set_decay_mask(self, decay) -> None:
        """decay: one entry per tensor, non-zero = weight decay applies; None = everywhere."""
        if decay is None:
            _check(self._L.bca_plan_set_decay_mask(self._h, None))
            return
        a = np.ascontiguousarray(decay, dtype=np.uint8)
        if a.shape != (self.n_tensors,):
            raise ValueError(f"expected {self.n_tensors} mask entries, got {a.shape}")
        buf = (C.c_uint8 * max(1, self.n_tensors)).from_buffer_copy(a.tobytes() or b"\0")
        _check(self._L.bca_plan_set_decay_mask(self._h, buf))

    def set_device_hyper(self, dev) -> None:
        """dev: a device buffer holding a bca_adam_device (see pack_device_hyper), or None for host arguments.
        While set, the compute calls take hyper-parameters and step from there (hp may be None)."""
        _check(self._L.bca_plan_set_device_hyper(self._h, _ptr(dev)))
        self._hyper_dev = dev                                  # keep the buffer alive while set

    # -- per-kernel timing of the fused call
    def profile(self, max_calls: int) -> None:
        _check(self._L.bca_plan_profile(self._h, max_calls))

    def profile_read(self):
        """(ms_sqnorm, ms_finalize, ms_adam) summed over n_calls, and n_calls; with the single pipelined launch
        (ms_finish_kernel, 0, ms_step_kernel)."""
        ms = (C.c_double * 3)()
        n = C.c_uint32()
        _check(self._L.bca_plan_profile_read(self._h, ms, C.byref(n)))
        return (ms[0], ms[1], ms[2]), int(n.value)

    def wait_stats(self):
        """(items that had to wait for their bucket's coefficient, polls they made) since the last call; synchronises."""
        out = (C.c_uint64 * 2)()
        _check(self._L.bca_plan_wait_stats(self._h, out))
        return int(out[0]), int(out[1])

    # -- compute (same names as the C ABI)
    def bucket_clip_norms(self, b0: int, b1: int, norms, stream=None) -> None:
        _check(self._L.bucket_clip_norms(self._h, b0, b1, _ptr(norms), _stream(stream)))

    def bucket_clip_apply(self, b0: int, b1: int, thresholds, norms, coefs=None, status=None, stream=None) -> None:
        _check(self._L.bucket_clip_apply(self._h, b0, b1, _ptr(thresholds), _ptr(norms), _ptr(coefs), _ptr(status),
                                         _stream(stream)))

    def bucket_clip(self, b0: int, b1: int, thresholds, norms=None, coefs=None, status=None, stream=None) -> None:
        _check(self._L.bucket_clip(self._h, b0, b1, _ptr(thresholds), _ptr(norms), _ptr(coefs), _ptr(status),
                                   _stream(stream)))

    def adam_step(self, hp: Optional[AdamHyper], step: int, stream=None) -> None:
        _check(self._L.adam_step(self._h, _hp(hp), step, _stream(stream)))

    def bucket_clip_adam(self, thresholds, hp: Optional[AdamHyper], step: int, flags: int = 0, norms=None, coefs=None,
                         status=None, stream=None) -> None:
        _check(self._L.bucket_clip_adam(self._h, _ptr(thresholds), _hp(hp), step, flags, _ptr(norms), _ptr(coefs),
                                        _ptr(status), _stream(stream)))

    def lamb_step(self, hp: Optional[AdamHyper], step: int, trust=None, stream=None) -> None:
        _check(self._L.lamb_step(self._h, _hp(hp), step, _ptr(trust), _stream(stream)))

    def bucket_clip_lamb(self, thresholds, hp: Optional[AdamHyper], step: int, flags: int = 0, norms=None, coefs=None,
                         trust=None, status=None, stream=None) -> None:
        _check(self._L.bucket_clip_lamb(self._h, _ptr(thresholds), _hp(hp), step, flags, _ptr(norms), _ptr(coefs),
                                        _ptr(trust), _ptr(status), _stream(stream)))
