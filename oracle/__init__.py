"""CPU oracle of the 8-bit optimizer step -- TEST INFRASTRUCTURE.

Thin numpy/ctypes front end of oracle/q8_oracle.c (the arithmetic lives there).
Only tests/, the smoke check and the benchmark's cpu_baseline leg may import it;
it imports nothing from the HIP package.
"""
from __future__ import annotations

import ctypes as C

import numpy as np

from .build import build as _build

FLAG_BIAS_CORRECTION = 1
FLAG_DECOUPLED_WD = 2

_lib = None


def bind(L):
    """Declare the argument types of the oracle's functions on a loaded library."""
    fp, u8p, i64, i32, f32 = C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_float
    L.oracle_build_codebook.argtypes = [i32, fp]
    L.oracle_nearest_code.argtypes = [fp, f32]
    L.oracle_nearest_code_bruteforce.argtypes = [fp, f32]
    L.oracle_quantize_blockwise.argtypes = [fp, fp, i64, i32, u8p, fp]
    L.oracle_dequantize_blockwise.argtypes = [fp, u8p, fp, i64, i32, fp]
    L.oracle_adam32_step.argtypes = [fp, fp, fp, fp, i64, f32, f32, f32, f32, f32, i64, i32]
    L.oracle_sgd32_step.argtypes = [fp, fp, fp, i64, f32, f32, f32]
    L.oracle_adam_scalars.argtypes = [f32, f32, f32, f32, f32, i64, i32, fp]
    L.oracle_adam8bit_step.argtypes = [fp, fp, u8p, u8p, fp, fp, fp, fp, i64, i32,
                                       f32, f32, f32, f32, f32, i64, i32]
    L.oracle_sgd8bit_step.argtypes = [fp, fp, u8p, fp, fp, i64, i32, f32, f32, f32]
    L.oracle_adam8bit_block_normalized.argtypes = [fp, fp, u8p, u8p, f32, f32, fp, fp, i32,
                                                   f32, f32, f32, f32, f32, i64, i32, fp, fp]
    L.oracle_adam8bit_step_bf16.argtypes = L.oracle_adam8bit_step.argtypes
    L.oracle_sgd8bit_step_bf16.argtypes = L.oracle_sgd8bit_step.argtypes
    L.oracle_adam8bit_step_f16.argtypes = L.oracle_adam8bit_step.argtypes
    L.oracle_sgd8bit_step_f16.argtypes = L.oracle_sgd8bit_step.argtypes
    L.oracle_f16_to_f32.argtypes = [C.c_uint16]; L.oracle_f16_to_f32.restype = f32
    L.oracle_f32_to_f16.argtypes = [f32]; L.oracle_f32_to_f16.restype = C.c_uint16
    L.oracle_bf16_to_f32.argtypes = [C.c_uint16]; L.oracle_bf16_to_f32.restype = f32
    L.oracle_f32_to_bf16.argtypes = [f32]; L.oracle_f32_to_bf16.restype = C.c_uint16
    for name in ("oracle_build_codebook", "oracle_nearest_code", "oracle_nearest_code_bruteforce",
                 "oracle_quantize_blockwise", "oracle_dequantize_blockwise", "oracle_adam32_step",
                 "oracle_sgd32_step", "oracle_adam_scalars", "oracle_adam8bit_step", "oracle_sgd8bit_step",
                 "oracle_adam8bit_step_bf16", "oracle_sgd8bit_step_bf16",
                 "oracle_adam8bit_step_f16", "oracle_sgd8bit_step_f16",
                 "oracle_adam8bit_block_normalized"):
        getattr(L, name).restype = i32
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = bind(C.CDLL(_build()))
    return _lib


def _p(a: np.ndarray, dtype) -> int:
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data


def _ok(rc):
    if rc != 0:
        raise ValueError("oracle call failed with status %d" % rc)


def nblocks(n: int, B: int) -> int:
    return (n + B - 1) // B


def build_codebook(is_signed: bool) -> np.ndarray:
    q = np.empty(256, np.float32)
    _ok(lib().oracle_build_codebook(int(bool(is_signed)), _p(q, np.float32)))
    return q


def nearest_code(q: np.ndarray, x) -> int:
    return lib().oracle_nearest_code(_p(q, np.float32), float(np.float32(x)))


def nearest_code_bruteforce(q: np.ndarray, x) -> int:
    return lib().oracle_nearest_code_bruteforce(_p(q, np.float32), float(np.float32(x)))


def quantize_blockwise(q, T, B):
    n = T.size
    TQ = np.empty(n, np.uint8)
    N = np.empty(nblocks(n, B), np.float32)
    _ok(lib().oracle_quantize_blockwise(_p(q, np.float32), _p(T, np.float32), n, B,
                                        _p(TQ, np.uint8), _p(N, np.float32)))
    return TQ, N


def dequantize_blockwise(q, TQ, N, B):
    n = TQ.size
    assert N.size == nblocks(n, B)
    TD = np.empty(n, np.float32)
    _ok(lib().oracle_dequantize_blockwise(_p(q, np.float32), _p(TQ, np.uint8), _p(N, np.float32), n, B,
                                          _p(TD, np.float32)))
    return TD


def adam32_step(w, g, m, r, alpha, beta1, beta2, eps, wd=0.0, t=1, flags=0):
    """In place on w, m, r."""
    n = w.size
    assert g.size == n and m.size == n and r.size == n
    _ok(lib().oracle_adam32_step(_p(w, np.float32), _p(g, np.float32), _p(m, np.float32), _p(r, np.float32),
                                 n, alpha, beta1, beta2, eps, wd, t, flags))


def adam_scalars(alpha, beta1, beta2, eps, wd=0.0, t=1, flags=0) -> dict:
    """The binary32 scalars the Adam step derives from its hyper-parameters."""
    out = np.empty(5, np.float32)
    _ok(lib().oracle_adam_scalars(alpha, beta1, beta2, eps, wd, t, flags, _p(out, np.float32)))
    return dict(omb1=out[0], omb2=out[1], alpha_t=out[2], isbc2=out[3], alpha_wd=out[4])


def sgd32_step(w, g, m, alpha, beta, wd=0.0):
    n = w.size
    assert g.size == n and m.size == n
    _ok(lib().oracle_sgd32_step(_p(w, np.float32), _p(g, np.float32), _p(m, np.float32), n, alpha, beta, wd))


def adam8bit_step(w, g, m_q, r_q, N_m, N_r, q_signed, q_unsigned, B,
                  alpha, beta1, beta2, eps, wd=0.0, t=1, flags=0):
    """In place on w, m_q, r_q, N_m, N_r."""
    n = w.size
    assert g.size == n and m_q.size == n and r_q.size == n
    assert N_m.size == nblocks(n, B) and N_r.size == nblocks(n, B)
    _ok(lib().oracle_adam8bit_step(_p(w, np.float32), _p(g, np.float32), _p(m_q, np.uint8), _p(r_q, np.uint8),
                                   _p(N_m, np.float32), _p(N_r, np.float32),
                                   _p(q_signed, np.float32), _p(q_unsigned, np.float32), n, B,
                                   alpha, beta1, beta2, eps, wd, t, flags))


def adam8bit_block_normalized(w, g, m_q, r_q, N_m, N_r, q_signed, q_unsigned,
                              alpha, beta1, beta2, eps, wd=0.0, t=1, flags=0):
    """Normalized new states (m / N_m', r / N_r') of one block, as the 8-bit Adam step forms them
    before the nearest-value search.  Inputs are the block's slices and its two old maxima."""
    n = w.size
    assert g.size == n and m_q.size == n and r_q.size == n
    x = np.empty(n, np.float32); y = np.empty(n, np.float32)
    _ok(lib().oracle_adam8bit_block_normalized(_p(w, np.float32), _p(g, np.float32), _p(m_q, np.uint8), _p(r_q, np.uint8),
                                               float(N_m), float(N_r), _p(q_signed, np.float32), _p(q_unsigned, np.float32),
                                               n, alpha, beta1, beta2, eps, wd, t, flags, _p(x, np.float32), _p(y, np.float32)))
    return x, y


def sgd8bit_step(w, g, m_q, N_m, q_signed, B, alpha, beta, wd=0.0):
    n = w.size
    assert g.size == n and m_q.size == n and N_m.size == nblocks(n, B)
    _ok(lib().oracle_sgd8bit_step(_p(w, np.float32), _p(g, np.float32), _p(m_q, np.uint8), _p(N_m, np.float32),
                                  _p(q_signed, np.float32), n, B, alpha, beta, wd))


# ------------------------------------------------------------------ bfloat16 storage of w and g
def bf16_to_f32(h) -> float:
    return float(lib().oracle_bf16_to_f32(int(h)))


def f32_to_bf16(x) -> int:
    return int(lib().oracle_f32_to_bf16(float(np.float32(x))))


def f16_to_f32(h) -> float:
    return float(lib().oracle_f16_to_f32(int(h)))


def f32_to_f16(x) -> int:
    return int(lib().oracle_f32_to_f16(float(np.float32(x))))


def adam8bit_step_f16(w, g, m_q, r_q, N_m, N_r, q_signed, q_unsigned, B,
                      alpha, beta1, beta2, eps, wd=0.0, t=1, flags=0):
    """w, g: uint16 arrays holding IEEE binary16 patterns.  In place on w, m_q, r_q, N_m, N_r."""
    n = w.size
    assert g.size == n and m_q.size == n and r_q.size == n
    assert N_m.size == nblocks(n, B) and N_r.size == nblocks(n, B)
    _ok(lib().oracle_adam8bit_step_f16(_p(w, np.uint16), _p(g, np.uint16), _p(m_q, np.uint8), _p(r_q, np.uint8),
                                       _p(N_m, np.float32), _p(N_r, np.float32),
                                       _p(q_signed, np.float32), _p(q_unsigned, np.float32), n, B,
                                       alpha, beta1, beta2, eps, wd, t, flags))


def sgd8bit_step_f16(w, g, m_q, N_m, q_signed, B, alpha, beta, wd=0.0):
    n = w.size
    assert g.size == n and m_q.size == n and N_m.size == nblocks(n, B)
    _ok(lib().oracle_sgd8bit_step_f16(_p(w, np.uint16), _p(g, np.uint16), _p(m_q, np.uint8), _p(N_m, np.float32),
                                      _p(q_signed, np.float32), n, B, alpha, beta, wd))


def adam8bit_step_bf16(w, g, m_q, r_q, N_m, N_r, q_signed, q_unsigned, B,
                       alpha, beta1, beta2, eps, wd=0.0, t=1, flags=0):
    """w, g: uint16 arrays holding bfloat16 patterns.  In place on w, m_q, r_q, N_m, N_r."""
    n = w.size
    assert g.size == n and m_q.size == n and r_q.size == n
    assert N_m.size == nblocks(n, B) and N_r.size == nblocks(n, B)
    _ok(lib().oracle_adam8bit_step_bf16(_p(w, np.uint16), _p(g, np.uint16), _p(m_q, np.uint8), _p(r_q, np.uint8),
                                        _p(N_m, np.float32), _p(N_r, np.float32),
                                        _p(q_signed, np.float32), _p(q_unsigned, np.float32), n, B,
                                        alpha, beta1, beta2, eps, wd, t, flags))


def sgd8bit_step_bf16(w, g, m_q, N_m, q_signed, B, alpha, beta, wd=0.0):
    n = w.size
    assert g.size == n and m_q.size == n and N_m.size == nblocks(n, B)
    _ok(lib().oracle_sgd8bit_step_bf16(_p(w, np.uint16), _p(g, np.uint16), _p(m_q, np.uint8), _p(N_m, np.float32),
                                       _p(q_signed, np.float32), n, B, alpha, beta, wd))
