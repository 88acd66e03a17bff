"""ctypes binding of libq8opt.so: same names as include/q8opt.h, argument marshalling only.

PyTorch appears here only as the owner of device memory and streams: functions take
torch CUDA tensors (or raw integer device addresses), check dtype/contiguity, and pass
`data_ptr()` plus the current HIP stream to the C ABI.  There is no CPU fallback: if the
library is missing, or a call returns an error status, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libq8opt.so")

FLAG_BIAS_CORRECTION = 1
FLAG_DECOUPLED_WD = 2

OK, EINVAL, EALIGN, EBLOCK, ELAUNCH, ENOMEM, ECODEBOOK, ELIMIT = 0, -1, -2, -3, -4, -5, -6, -7

EXPORTS = (
    "q8_status_str", "q8_build_codebook", "q8_qtable_bytes", "q8_build_qtable", "q8_host_nearest_code",
    "q8_quantize_blockwise", "q8_dequantize_blockwise", "q8_adam8bit_step", "q8_sgd8bit_step",
    "q8_plan_create", "q8_plan_destroy", "q8_multi_adam8bit_step", "q8_multi_sgd8bit_step",
    "q8_adam8bit_step_bf16", "q8_sgd8bit_step_bf16", "q8_plan_create_bf16",
    "q8_adam8bit_step_f16", "q8_sgd8bit_step_f16", "q8_plan_create_f16",
    "q8_multi_adam8bit_step_noalloc",
)


class Q8Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s" % (where, status_str(status)))


class q8_tensor(C.Structure):
    _fields_ = [("w", C.c_void_p), ("g", C.c_void_p), ("n", C.c_int64),
                ("m_q", C.c_void_p), ("r_q", C.c_void_p), ("N_m", C.c_void_p), ("N_r", C.c_void_p),
                ("m_f32", C.c_void_p), ("r_f32", C.c_void_p)]


_lib = None


def lib():
    """Load libq8opt.so (built by `python -m paper_2412_01195_amd.build` or __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libq8opt.so is not built (%s); run __graft_entry__.build()" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, f32 = C.c_void_p, C.c_int64, C.c_int, C.c_float
        L.q8_status_str.argtypes = [i32]; L.q8_status_str.restype = C.c_char_p
        L.q8_build_codebook.argtypes = [i32, vp]
        L.q8_qtable_bytes.argtypes = []; L.q8_qtable_bytes.restype = C.c_size_t
        L.q8_build_qtable.argtypes = [vp, vp]
        L.q8_host_nearest_code.argtypes = [vp, f32]
        L.q8_quantize_blockwise.argtypes = [vp, vp, i64, i32, vp, vp, vp]
        L.q8_dequantize_blockwise.argtypes = [vp, vp, vp, i64, i32, vp, vp]
        L.q8_adam8bit_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i32, f32, f32, f32, f32, f32, i64, i32, vp]
        L.q8_sgd8bit_step.argtypes = [vp, vp, vp, vp, vp, i64, i32, f32, f32, f32, vp]
        L.q8_adam8bit_step_bf16.argtypes = L.q8_adam8bit_step.argtypes
        L.q8_sgd8bit_step_bf16.argtypes = L.q8_sgd8bit_step.argtypes
        L.q8_adam8bit_step_f16.argtypes = L.q8_adam8bit_step.argtypes
        L.q8_sgd8bit_step_f16.argtypes = L.q8_sgd8bit_step.argtypes
        L.q8_plan_create.argtypes = [C.POINTER(q8_tensor), i32, i32, C.POINTER(vp)]
        L.q8_plan_create_bf16.argtypes = L.q8_plan_create.argtypes
        L.q8_plan_create_f16.argtypes = L.q8_plan_create.argtypes
        L.q8_plan_destroy.argtypes = [vp]
        L.q8_multi_adam8bit_step.argtypes = [vp, vp, vp, f32, f32, f32, f32, f32, i64, i32, vp]
        L.q8_multi_sgd8bit_step.argtypes = [vp, vp, f32, f32, f32, vp]
        L.q8_multi_adam8bit_step_noalloc.argtypes = [C.POINTER(q8_tensor), i32, i32, vp, vp,
                                                     f32, f32, f32, f32, f32, i64, i32, vp]
        for name in EXPORTS:
            if name not in ("q8_status_str", "q8_qtable_bytes"):
                getattr(L, name).restype = i32
        _lib = L
    return _lib


def status_str(status: int) -> str:
    return lib().q8_status_str(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise Q8Error(status, where)


# ----------------------------------------------------------------------------- host side
def build_codebook(is_signed: bool) -> np.ndarray:
    q = np.empty(256, np.float32)
    _check(lib().q8_build_codebook(int(bool(is_signed)), q.ctypes.data), "q8_build_codebook")
    return q


def qtable_bytes() -> int:
    return int(lib().q8_qtable_bytes())


def build_qtable(qmap: np.ndarray) -> np.ndarray:
    """Host blob (uint8 array) to be copied to 16-byte aligned device memory."""
    qmap = np.ascontiguousarray(qmap, np.float32)
    if qmap.shape != (256,):
        raise ValueError("qmap must hold 256 values")
    blob = np.zeros(qtable_bytes(), np.uint8)
    _check(lib().q8_build_qtable(qmap.ctypes.data, blob.ctypes.data), "q8_build_qtable")
    return blob


def host_nearest_code(qtable: np.ndarray, x) -> int:
    assert qtable.dtype == np.uint8 and qtable.size == qtable_bytes()
    c = lib().q8_host_nearest_code(qtable.ctypes.data, float(np.float32(x)))
    if c < 0:
        raise Q8Error(c, "q8_host_nearest_code")
    return c


# ----------------------------------------------------------------------------- device side
def _ptrs(*specs):
    """Device addresses of torch CUDA tensors; a spec is (tensor | int | None, dtype name,
    elements the call will touch, name).  Integers (raw device addresses) and None pass
    through.  The C ABI sees plain pointers and cannot check sizes, so a tensor of the wrong
    type or too small is refused here instead of being overrun on the device; types and sizes
    of all arguments are checked before their placement."""
    for t, dtype_name, need, what in specs:
        if t is None or isinstance(t, (int, np.integer)):
            continue
        if dtype_name is not None and str(t.dtype) != "torch." + dtype_name:
            raise ValueError("%s: expected dtype %s, got %s" % (what, dtype_name, t.dtype))
        if t.numel() < need:
            raise ValueError("%s holds %d elements, the call needs %d" % (what, t.numel(), need))
    out = []
    for t, dtype_name, need, what in specs:
        if t is None:
            out.append(0)
        elif isinstance(t, (int, np.integer)):
            out.append(int(t))
        elif not t.is_cuda or not t.is_contiguous():
            raise ValueError("%s: expected a contiguous CUDA tensor" % what)
        else:
            out.append(t.data_ptr())
    return out


def _blocks(n: int, B: int) -> int:
    return -(-n // B) if B > 0 else 0          # an invalid B is reported by the library (Q8_EBLOCK)


def _qtab(t, what: str):
    return (t, "uint8", qtable_bytes(), what)


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def upload_qtable(blob: np.ndarray, device="cuda"):
    """Copy a host qtable blob into a device uint8 tensor (torch allocations are 256-byte aligned)."""
    import torch
    return torch.from_numpy(blob).to(device)


def quantize_blockwise(qtable, T, B: int, TQ, N, n: Optional[int] = None):
    n = T.numel() if n is None else n
    q, t, tq, nn = _ptrs(_qtab(qtable, "qtable"), (T, "float32", n, "T"), (TQ, "uint8", n, "TQ"),
                         (N, "float32", _blocks(n, B), "N"))
    _check(lib().q8_quantize_blockwise(q, t, n, B, tq, nn, _stream()), "q8_quantize_blockwise")


def dequantize_blockwise(qtable, TQ, N, B: int, TD, n: Optional[int] = None):
    n = TQ.numel() if n is None else n
    q, tq, nn, td = _ptrs(_qtab(qtable, "qtable"), (TQ, "uint8", n, "TQ"), (N, "float32", _blocks(n, B), "N"),
                          (TD, "float32", n, "TD"))
    _check(lib().q8_dequantize_blockwise(q, tq, nn, n, B, td, _stream()), "q8_dequantize_blockwise")


def _adam(entry: str, wg_dtype: str, w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B,
          alpha, beta1, beta2, eps, weight_decay, t, flags, n):
    n = w.numel() if n is None else n
    nb = _blocks(n, B)
    p = _ptrs((w, wg_dtype, n, "w"), (g, wg_dtype, n, "g"), (m_q, "uint8", n, "m_q"), (r_q, "uint8", n, "r_q"),
              (N_m, "float32", nb, "N_m"), (N_r, "float32", nb, "N_r"),
              _qtab(qtable_signed, "qtable_signed"), _qtab(qtable_unsigned, "qtable_unsigned"))
    _check(getattr(lib(), entry)(*p, n, B, alpha, beta1, beta2, eps, weight_decay, t, flags, _stream()), entry)


def _sgd(entry: str, wg_dtype: str, w, g, m_q, N_m, qtable_signed, B, alpha, beta, weight_decay, n):
    n = w.numel() if n is None else n
    p = _ptrs((w, wg_dtype, n, "w"), (g, wg_dtype, n, "g"), (m_q, "uint8", n, "m_q"),
              (N_m, "float32", _blocks(n, B), "N_m"), _qtab(qtable_signed, "qtable_signed"))
    _check(getattr(lib(), entry)(*p, n, B, alpha, beta, weight_decay, _stream()), entry)


def adam8bit_step(w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B: int,
                  alpha, beta1, beta2, eps, weight_decay=0.0, t=1, flags=0, n: Optional[int] = None):
    _adam("q8_adam8bit_step", "float32", w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B,
          alpha, beta1, beta2, eps, weight_decay, t, flags, n)


def adam8bit_step_bf16(w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B: int,
                       alpha, beta1, beta2, eps, weight_decay=0.0, t=1, flags=0, n: Optional[int] = None):
    """w, g: torch.bfloat16 tensors."""
    _adam("q8_adam8bit_step_bf16", "bfloat16", w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B,
          alpha, beta1, beta2, eps, weight_decay, t, flags, n)


def adam8bit_step_f16(w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B: int,
                      alpha, beta1, beta2, eps, weight_decay=0.0, t=1, flags=0, n: Optional[int] = None):
    """w, g: torch.float16 tensors."""
    _adam("q8_adam8bit_step_f16", "float16", w, g, m_q, r_q, N_m, N_r, qtable_signed, qtable_unsigned, B,
          alpha, beta1, beta2, eps, weight_decay, t, flags, n)


def sgd8bit_step(w, g, m_q, N_m, qtable_signed, B: int, alpha, beta, weight_decay=0.0, n: Optional[int] = None):
    _sgd("q8_sgd8bit_step", "float32", w, g, m_q, N_m, qtable_signed, B, alpha, beta, weight_decay, n)


def sgd8bit_step_bf16(w, g, m_q, N_m, qtable_signed, B: int, alpha, beta, weight_decay=0.0,
                      n: Optional[int] = None):
    """w, g: torch.bfloat16 tensors."""
    _sgd("q8_sgd8bit_step_bf16", "bfloat16", w, g, m_q, N_m, qtable_signed, B, alpha, beta, weight_decay, n)


def sgd8bit_step_f16(w, g, m_q, N_m, qtable_signed, B: int, alpha, beta, weight_decay=0.0,
                     n: Optional[int] = None):
    """w, g: torch.float16 tensors."""
    _sgd("q8_sgd8bit_step_f16", "float16", w, g, m_q, N_m, qtable_signed, B, alpha, beta, weight_decay, n)


_FIELDS = (("w", None), ("g", None), ("m_q", "uint8"), ("r_q", "uint8"), ("N_m", "float32"), ("N_r", "float32"),
           ("m_f32", "float32"), ("r_f32", "float32"))


def _tensor_array(tensors: Sequence[dict], wg: str, B: int):
    specs = []
    for i, t in enumerate(tensors):
        n = t["w"].numel()
        for key, dt in _FIELDS:
            need = _blocks(n, B) if key in ("N_m", "N_r") else n
            specs.append((t.get(key), dt or wg, need, "tensor %d: %s" % (i, key)))
    ptrs = _ptrs(*specs)
    arr = (q8_tensor * len(tensors))()
    for i, t in enumerate(tensors):
        arr[i].n = t["w"].numel()
        for k, (key, _) in enumerate(_FIELDS):
            setattr(arr[i], key, ptrs[i * len(_FIELDS) + k])
    return arr


def multi_adam8bit_step_noalloc(tensors: Sequence[dict], B: int, qtable_signed, qtable_unsigned,
                                alpha, beta1, beta2, eps, weight_decay=0.0, t=1, flags=0):
    """q8_multi_adam8bit_step_noalloc: one Adam step over a list of fp32 tensors (dicts as for Plan)
    without a plan and without any device allocation by the library."""
    arr = _tensor_array(tensors, "float32", B)
    qs, qu = _ptrs(_qtab(qtable_signed, "qtable_signed"), _qtab(qtable_unsigned, "qtable_unsigned"))
    _check(lib().q8_multi_adam8bit_step_noalloc(arr, len(tensors), B, qs, qu, alpha, beta1, beta2, eps,
                                                weight_decay, t, flags, _stream()),
           "q8_multi_adam8bit_step_noalloc")


class Plan:
    """q8_plan: a list of parameter tensors updated by one launch.

    Each entry is a dict with keys w, g and either (m_q, N_m[, r_q, N_r]) or (m_f32[, r_f32]).
    wg_dtype: "float32" (default), "bfloat16" or "float16" = element type of every w and g
    (q8_plan_create, q8_plan_create_bf16, q8_plan_create_f16); bf16=True is short for "bfloat16"."""

    def __init__(self, tensors: Sequence[dict], B: int, bf16: bool = False, wg_dtype: Optional[str] = None):
        self._keep = list(tensors)
        wg = wg_dtype or ("bfloat16" if bf16 else "float32")
        if wg not in ("float32", "bfloat16", "float16"):
            raise ValueError("wg_dtype must be float32, bfloat16 or float16")
        arr = _tensor_array(tensors, wg, B)
        h = C.c_void_p()
        create = {"float32": lib().q8_plan_create, "bfloat16": lib().q8_plan_create_bf16,
                  "float16": lib().q8_plan_create_f16}[wg]
        _check(create(arr, len(tensors), B, C.byref(h)), "q8_plan_create")
        self._h = h

    def multi_adam8bit_step(self, qtable_signed, qtable_unsigned, alpha, beta1, beta2, eps,
                            weight_decay=0.0, t=1, flags=0):
        qs, qu = _ptrs(_qtab(qtable_signed, "qtable_signed"), _qtab(qtable_unsigned, "qtable_unsigned"))
        _check(lib().q8_multi_adam8bit_step(self._h, qs, qu,
                                            alpha, beta1, beta2, eps, weight_decay, t, flags, _stream()),
               "q8_multi_adam8bit_step")

    def multi_sgd8bit_step(self, qtable_signed, alpha, beta, weight_decay=0.0):
        qs, = _ptrs(_qtab(qtable_signed, "qtable_signed"))
        _check(lib().q8_multi_sgd8bit_step(self._h, qs, alpha, beta, weight_decay,
                                           _stream()), "q8_multi_sgd8bit_step")

    def destroy(self):
        if self._h:
            _check(lib().q8_plan_destroy(self._h), "q8_plan_destroy")
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
