"""ctypes binding of the CPU oracle (oracle/coat_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the bench's
cpu_baseline leg, never by the product package.  It holds no arithmetic of its own; every
function marshals numpy arrays into the C oracle.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "coat_ref.c")
_LIB = os.path.join(_HERE, "libcoat_ref.so")

FLAG_EXPAND, FLAG_M_E5M2, FLAG_E5M2, FLAG_V_E5M2, FLAG_M_PLAIN, FLAG_V_PLAIN, FLAG_BF16_SCALE, FLAG_BF16_K, FLAG_DQ_FP32 = 1, 2, 2, 4, 8, 16, 32, 64, 128


class HParams(ctypes.Structure):
    """Mirror of coat_ref_hparams."""

    _fields_ = [
        ("lr", ctypes.c_float),
        ("beta1", ctypes.c_float),
        ("beta2", ctypes.c_float),
        ("eps", ctypes.c_float),
        ("weight_decay", ctypes.c_float),
        ("step", ctypes.c_int32),
        ("group_size", ctypes.c_int32),
        ("flags", ctypes.c_uint32),
        ("k_min", ctypes.c_float),
        ("k_max", ctypes.c_float),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64 libm, OpenMP over groups)."""
    stale = (not os.path.exists(_LIB)
             or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
             or os.path.getmtime(_LIB) < os.path.getmtime(os.path.join(_HERE, "coat_ref.h")))
    if force or stale:
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        u8p = ctypes.POINTER(ctypes.c_uint8)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f32p = ctypes.POINTER(ctypes.c_float)
        f64p = ctypes.POINTER(ctypes.c_double)
        L.coat_ref_e4m3_decode.restype = ctypes.c_double
        L.coat_ref_e4m3_decode.argtypes = [ctypes.c_uint8]
        L.coat_ref_e4m3_encode.restype = ctypes.c_uint8
        L.coat_ref_e4m3_encode.argtypes = [ctypes.c_double]
        L.coat_ref_quant_group.restype = None
        L.coat_ref_quant_group.argtypes = [f32p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32,
                                           ctypes.c_float, ctypes.c_float, u8p, f32p, f32p]
        L.coat_ref_dequant_group.restype = None
        L.coat_ref_dequant_group.argtypes = [u8p, f32p, f32p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32, f32p]
        L.coat_ref_dequant_group_f64.restype = None
        L.coat_ref_dequant_group_f64.argtypes = [u8p, f32p, f32p, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32, f64p]
        for name in ("coat_ref_e5m2_decode", "coat_ref_e5m2_encode"):
            getattr(L, name)
        L.coat_ref_e5m2_decode.restype = ctypes.c_double
        L.coat_ref_e5m2_decode.argtypes = [ctypes.c_uint8]
        L.coat_ref_e5m2_encode.restype = ctypes.c_uint8
        L.coat_ref_e5m2_encode.argtypes = [ctypes.c_double]
        L.coat_ref_fp8_adamw_step.restype = ctypes.c_int
        L.coat_ref_fp8_adamw_step.argtypes = [f32p, u16p, u8p, f32p, f32p, u8p, f32p, f32p,
                                              ctypes.c_uint64, ctypes.POINTER(HParams)]
        L.coat_ref_fp8_adamw_step_bf16w.restype = ctypes.c_int
        L.coat_ref_fp8_adamw_step_bf16w.argtypes = [f32p, u16p, u16p, u8p, f32p, f32p, u8p, f32p, f32p,
                                                    ctypes.c_uint64, ctypes.POINTER(HParams)]
        L.coat_ref_act_quant_group.restype = None
        L.coat_ref_act_quant_group.argtypes = [u16p, ctypes.c_uint64, ctypes.c_int32, u8p, f32p]
        L.coat_ref_act_quant_tensor.restype = None
        L.coat_ref_act_quant_tensor.argtypes = [u16p, ctypes.c_uint64, ctypes.c_int32, f32p, f32p, u8p]
        L.coat_ref_num_threads.restype = ctypes.c_int
        L.coat_ref_num_threads.argtypes = []
        _lib = L
    return _lib


def _ptr(a: np.ndarray, dtype, ctype):
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(ctypes.POINTER(ctype))


def n_groups(n: int, G: int) -> int:
    return (n + G - 1) // G


def num_threads() -> int:
    return int(lib().coat_ref_num_threads())


def e4m3_decode(code: int) -> float:
    return float(lib().coat_ref_e4m3_decode(int(code) & 0xFF))


def e4m3_encode(q: float) -> int:
    return int(lib().coat_ref_e4m3_encode(float(q)))


def e5m2_decode(code: int) -> float:
    return float(lib().coat_ref_e5m2_decode(int(code) & 0xFF))


def e5m2_encode(q: float) -> int:
    return int(lib().coat_ref_e5m2_encode(float(q)))


def quant_group(x: np.ndarray, G: int, expand: bool = True, k_min: float = 0.0, k_max: float = 0.0,
                e5m2: bool = False, bf16_scale: bool = False, bf16_k: bool = False):
    """x: fp32 array (flattened).  Returns (codes u8 [n], scale f32 [ng], k f32 [ng]).
    bf16_scale / bf16_k: the scales / exponents are bf16 values (held in the float arrays)."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    n = x.size
    ng = n_groups(n, G)
    q = np.zeros(n, dtype=np.uint8)
    scale = np.zeros(ng, dtype=np.float32)
    k = np.ones(ng, dtype=np.float32)
    if n:
        lib().coat_ref_quant_group(_ptr(x, np.float32, ctypes.c_float), n, G,
                                   (FLAG_EXPAND if expand else 0) | (FLAG_E5M2 if e5m2 else 0)
                                   | (FLAG_BF16_SCALE if bf16_scale else 0) | (FLAG_BF16_K if bf16_k else 0),
                                   k_min, k_max,
                                   _ptr(q, np.uint8, ctypes.c_uint8),
                                   _ptr(scale, np.float32, ctypes.c_float),
                                   _ptr(k, np.float32, ctypes.c_float))
    return q, scale, k


def dequant_group(q: np.ndarray, scale: np.ndarray, k: np.ndarray, G: int, f64: bool = False,
                  e5m2: bool = False):
    flags = FLAG_E5M2 if e5m2 else 0
    q = np.ascontiguousarray(q, dtype=np.uint8).reshape(-1)
    scale = np.ascontiguousarray(scale, dtype=np.float32).reshape(-1)
    k = np.ascontiguousarray(k, dtype=np.float32).reshape(-1)
    n = q.size
    assert scale.size == n_groups(n, G) and k.size == scale.size
    if f64:
        x = np.zeros(n, dtype=np.float64)
        if n:
            lib().coat_ref_dequant_group_f64(_ptr(q, np.uint8, ctypes.c_uint8),
                                             _ptr(scale, np.float32, ctypes.c_float),
                                             _ptr(k, np.float32, ctypes.c_float), n, G, flags,
                                             _ptr(x, np.float64, ctypes.c_double))
        return x
    x = np.zeros(n, dtype=np.float32)
    if n:
        lib().coat_ref_dequant_group(_ptr(q, np.uint8, ctypes.c_uint8),
                                     _ptr(scale, np.float32, ctypes.c_float),
                                     _ptr(k, np.float32, ctypes.c_float), n, G, flags,
                                     _ptr(x, np.float32, ctypes.c_float))
    return x


def act_quant_group(x_bf16: np.ndarray, G: int):
    """bf16 bit patterns [n] -> (codes u8 [n], scale f32 [ng])."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16).reshape(-1)
    n = x.size
    q = np.zeros(n, np.uint8)
    scale = np.zeros(n_groups(n, G), np.float32)
    if n:
        lib().coat_ref_act_quant_group(_ptr(x, np.uint16, ctypes.c_uint16), n, G,
                                       _ptr(q, np.uint8, ctypes.c_uint8), _ptr(scale, np.float32, ctypes.c_float))
    return q, scale


def act_quant_tensor(x_bf16: np.ndarray, G: int):
    """Group Scaling: bf16 bit patterns [n] -> (codes u8 [n], tensor scale f32, group_amax f32 [ng])."""
    x = np.ascontiguousarray(x_bf16, dtype=np.uint16).reshape(-1)
    n = x.size
    q = np.zeros(n, np.uint8)
    amax = np.zeros(n_groups(n, G), np.float32)
    ts = np.zeros(1, np.float32)
    if n:
        lib().coat_ref_act_quant_tensor(_ptr(x, np.uint16, ctypes.c_uint16), n, G,
                                        _ptr(amax, np.float32, ctypes.c_float), _ptr(ts, np.float32, ctypes.c_float),
                                        _ptr(q, np.uint8, ctypes.c_uint8))
    return q, float(ts[0]), amax


def step_flags(expand=True, m_e5m2=False, v_e5m2=False, m_plain=False, v_plain=False, bf16_scale=False,
               bf16_k=False) -> int:
    return ((FLAG_EXPAND if expand else 0) | (FLAG_M_E5M2 if m_e5m2 else 0) | (FLAG_V_E5M2 if v_e5m2 else 0)
            | (FLAG_M_PLAIN if m_plain else 0) | (FLAG_V_PLAIN if v_plain else 0)
            | (FLAG_BF16_SCALE if bf16_scale else 0) | (FLAG_BF16_K if bf16_k else 0))


def make_hparams(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1,
                 group_size=128, expand=True, k_min=0.0, k_max=0.0,
                 m_e5m2=False, v_e5m2=False, m_plain=False, v_plain=False, bf16_scale=False, bf16_k=False) -> HParams:
    return HParams(lr, beta1, beta2, eps, weight_decay, int(step), int(group_size),
                   step_flags(expand, m_e5m2, v_e5m2, m_plain, v_plain, bf16_scale, bf16_k), k_min, k_max)


def fp8_adamw_step(w, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, hp: HParams, w_bf16=None) -> int:
    """In-place step on numpy arrays.  grad_bf16 holds raw bf16 bit patterns (uint16).
    w_bf16 (uint16 [n], optional): receives the new weights rounded to bf16."""
    n = w.size
    if w_bf16 is not None:
        assert w_bf16.size == n
        return int(lib().coat_ref_fp8_adamw_step_bf16w(
            _ptr(w, np.float32, ctypes.c_float), _ptr(w_bf16, np.uint16, ctypes.c_uint16),
            _ptr(grad_bf16, np.uint16, ctypes.c_uint16),
            _ptr(m_q, np.uint8, ctypes.c_uint8), _ptr(m_scale, np.float32, ctypes.c_float),
            _ptr(m_k, np.float32, ctypes.c_float),
            _ptr(v_q, np.uint8, ctypes.c_uint8), _ptr(v_scale, np.float32, ctypes.c_float),
            _ptr(v_k, np.float32, ctypes.c_float), n, ctypes.byref(hp)))
    ng = n_groups(n, hp.group_size)
    assert grad_bf16.size == n and m_q.size == n and v_q.size == n
    for a in (m_scale, m_k, v_scale, v_k):
        assert a.size == ng
    return int(lib().coat_ref_fp8_adamw_step(
        _ptr(w, np.float32, ctypes.c_float), _ptr(grad_bf16, np.uint16, ctypes.c_uint16),
        _ptr(m_q, np.uint8, ctypes.c_uint8), _ptr(m_scale, np.float32, ctypes.c_float),
        _ptr(m_k, np.float32, ctypes.c_float),
        _ptr(v_q, np.uint8, ctypes.c_uint8), _ptr(v_scale, np.float32, ctypes.c_float),
        _ptr(v_k, np.float32, ctypes.c_float), n, ctypes.byref(hp)))


if __name__ == "__main__":
    print(build(force=True))
