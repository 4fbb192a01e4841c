"""Thin ctypes binding of the C ABI in include/coat.h.

Argument marshalling only: every arithmetic step runs in the HIP kernels.  Tensors are
torch CUDA (ROCm) tensors used purely as owners of device memory; the kernels run on
torch's current stream.  There is no CPU fallback: without the built library, or with
host tensors, the calls raise.
"""
from __future__ import annotations

import ctypes
import os

from . import build as _build

FLAG_EXPAND, FLAG_M_E5M2, FLAG_E5M2, FLAG_V_E5M2, FLAG_M_PLAIN, FLAG_V_PLAIN = 1, 2, 2, 4, 8, 16
SUPPORTED_GROUP_SIZES = (32, 64, 128, 256, 512)

ACT_GROUP_SIZES = (16,) + SUPPORTED_GROUP_SIZES
ACT_WORKSPACE_FLOATS = 64

EXPORTS = ("coat_fp8_adamw_step", "coat_fp8_adamw_step_bf16w", "coat_quant_group", "coat_dequant_group",
           "coat_act_quant_group", "coat_act_quant_tensor", "coat_act_quant_tensor_from_group_amax",
           "coat_strerror", "coat_version")


class CoatError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("coat error %d: %s" % (code, text))
        self.code = code


class HParams(ctypes.Structure):
    """Mirror of coat_adamw_hparams."""

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


def step_flags(expand=True, m_e5m2=False, v_e5m2=False, m_plain=False, v_plain=False) -> int:
    return ((FLAG_EXPAND if expand else 0) | (FLAG_M_E5M2 if m_e5m2 else 0) | (FLAG_V_E5M2 if v_e5m2 else 0)
            | (FLAG_M_PLAIN if m_plain else 0) | (FLAG_V_PLAIN if v_plain else 0))


def make_hparams(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1,
                 group_size=128, expand=True, k_min=0.0, k_max=0.0,
                 m_e5m2=False, v_e5m2=False, m_plain=False, v_plain=False) -> HParams:
    return HParams(lr, beta1, beta2, eps, weight_decay, int(step), int(group_size),
                   step_flags(expand, m_e5m2, v_e5m2, m_plain, v_plain), k_min, k_max)


_lib = None


def lib():
    """Load libcoat.so (built beforehand by build.build()); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            raise RuntimeError("libcoat.so is not built: run `python -m paper_2410_19313_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(_build.LIB)
        vp = ctypes.c_void_p
        L.coat_fp8_adamw_step.restype = ctypes.c_int
        L.coat_fp8_adamw_step.argtypes = [vp] * 8 + [ctypes.c_uint64, ctypes.POINTER(HParams), vp]
        L.coat_fp8_adamw_step_bf16w.restype = ctypes.c_int
        L.coat_fp8_adamw_step_bf16w.argtypes = [vp] * 9 + [ctypes.c_uint64, ctypes.POINTER(HParams), vp]
        L.coat_quant_group.restype = ctypes.c_int
        L.coat_quant_group.argtypes = [vp, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32,
                                       ctypes.c_float, ctypes.c_float, vp, vp, vp, vp]
        L.coat_dequant_group.restype = ctypes.c_int
        L.coat_dequant_group.argtypes = [vp, vp, vp, ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32, vp, vp]
        L.coat_act_quant_group.restype = ctypes.c_int
        L.coat_act_quant_group.argtypes = [vp, ctypes.c_uint64, ctypes.c_int32, vp, vp, vp]
        for f in (L.coat_act_quant_tensor, L.coat_act_quant_tensor_from_group_amax):
            f.restype = ctypes.c_int
            f.argtypes = [vp, ctypes.c_uint64, ctypes.c_int32, vp, vp, vp, vp, vp, vp]
        L.coat_strerror.restype = ctypes.c_char_p
        L.coat_strerror.argtypes = [ctypes.c_int]
        L.coat_version.restype = ctypes.c_int
        L.coat_version.argtypes = []
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().coat_strerror(int(code)).decode()


def _check(rc: int):
    if rc != 0:
        raise CoatError(rc, strerror(rc))


def _dev_ptr(t, dtype, numel=None):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("expected a device tensor (this library has no host path)")
    if t.dtype != dtype:
        raise TypeError("expected dtype %s, got %s" % (dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    if numel is not None and t.numel() != numel:
        raise ValueError("expected %d elements, got %d" % (numel, t.numel()))
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def n_groups(n: int, G: int) -> int:
    return (n + G - 1) // G


def coat_fp8_adamw_step(w, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, hp: HParams) -> None:
    """In-place fused step.  w fp32 [n]; grad_bf16 bfloat16 [n]; m_q/v_q uint8 [n];
    *_scale/*_k fp32 [ceil(n/G)].  Asynchronous on torch's current stream."""
    import torch
    n = w.numel()
    ng = n_groups(n, hp.group_size) if hp.group_size > 0 else 0
    _check(lib().coat_fp8_adamw_step(
        _dev_ptr(w, torch.float32), _dev_ptr(grad_bf16, torch.bfloat16, n),
        _dev_ptr(m_q, torch.uint8, n), _dev_ptr(m_scale, torch.float32, ng), _dev_ptr(m_k, torch.float32, ng),
        _dev_ptr(v_q, torch.uint8, n), _dev_ptr(v_scale, torch.float32, ng), _dev_ptr(v_k, torch.float32, ng),
        n, ctypes.byref(hp), _stream()))


def coat_fp8_adamw_step_bf16w(w, w_bf16, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, hp: HParams) -> None:
    """coat_fp8_adamw_step that also writes the new weights as bfloat16 into w_bf16 [n]."""
    import torch
    n = w.numel()
    ng = n_groups(n, hp.group_size) if hp.group_size > 0 else 0
    _check(lib().coat_fp8_adamw_step_bf16w(
        _dev_ptr(w, torch.float32), _dev_ptr(w_bf16, torch.bfloat16, n), _dev_ptr(grad_bf16, torch.bfloat16, n),
        _dev_ptr(m_q, torch.uint8, n), _dev_ptr(m_scale, torch.float32, ng), _dev_ptr(m_k, torch.float32, ng),
        _dev_ptr(v_q, torch.uint8, n), _dev_ptr(v_scale, torch.float32, ng), _dev_ptr(v_k, torch.float32, ng),
        n, ctypes.byref(hp), _stream()))


def coat_quant_group(x, G: int, expand: bool = True, k_min: float = 0.0, k_max: float = 0.0,
                     out=None, e5m2: bool = False):
    """x fp32 [n] -> (codes uint8 [n], scale fp32 [ng], k fp32 [ng]) written on the device."""
    import torch
    n = x.numel()
    ng = n_groups(n, G) if G > 0 else 0
    if out is None:
        out = (torch.empty(n, dtype=torch.uint8, device=x.device),
               torch.empty(ng, dtype=torch.float32, device=x.device),
               torch.empty(ng, dtype=torch.float32, device=x.device))
    q, scale, k = out
    _check(lib().coat_quant_group(_dev_ptr(x, torch.float32), n, G,
                                  (FLAG_EXPAND if expand else 0) | (FLAG_E5M2 if e5m2 else 0),
                                  k_min, k_max, _dev_ptr(q, torch.uint8, n),
                                  _dev_ptr(scale, torch.float32, ng), _dev_ptr(k, torch.float32, ng),
                                  _stream()))
    return q, scale, k


def coat_dequant_group(q, scale, k, G: int, out=None, e5m2: bool = False):
    """codes uint8 [n] + per-group scale, k -> fp32 [n] on the device."""
    import torch
    n = q.numel()
    ng = n_groups(n, G) if G > 0 else 0
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=q.device)
    _check(lib().coat_dequant_group(_dev_ptr(q, torch.uint8), _dev_ptr(scale, torch.float32, ng),
                                    _dev_ptr(k, torch.float32, ng), n, G, FLAG_E5M2 if e5m2 else 0,
                                    _dev_ptr(out, torch.float32, n), _stream()))
    return out


def coat_act_quant_group(x_bf16, G: int = 16, out=None):
    """x bfloat16 [n] -> (codes uint8 [n], scale fp32 [ng]): the 1xG activation quantizer."""
    import torch
    n = x_bf16.numel()
    ng = n_groups(n, G) if G > 0 else 0
    if out is None:
        out = (torch.empty(n, dtype=torch.uint8, device=x_bf16.device),
               torch.empty(ng, dtype=torch.float32, device=x_bf16.device))
    q, scale = out
    _check(lib().coat_act_quant_group(_dev_ptr(x_bf16, torch.bfloat16), n, G, _dev_ptr(q, torch.uint8, n),
                                      _dev_ptr(scale, torch.float32, ng), _stream()))
    return q, scale


def act_workspace(device):
    """Scratch for the per-tensor quantizer's stage 2 (contents undefined; one per concurrent call)."""
    import torch
    return torch.empty(ACT_WORKSPACE_FLOATS, dtype=torch.float32, device=device)


def coat_act_quant_tensor(x_bf16, G: int = 16, out=None, workspace=None):
    """x bfloat16 [n] -> (codes uint8 [n], tensor_scale fp32 [1], group_amax fp32 [ng], tensor_amax fp32 [1]):
    per-tensor quantization with Group Scaling's two-stage max."""
    import torch
    n = x_bf16.numel()
    ng = n_groups(n, G) if G > 0 else 0
    dev = x_bf16.device
    if out is None:
        out = (torch.empty(n, dtype=torch.uint8, device=dev), torch.empty(1, dtype=torch.float32, device=dev),
               torch.empty(ng, dtype=torch.float32, device=dev), torch.empty(1, dtype=torch.float32, device=dev))
    if workspace is None:
        workspace = act_workspace(dev)
    q, tscale, gamax, tamax = out
    _check(lib().coat_act_quant_tensor(_dev_ptr(x_bf16, torch.bfloat16), n, G, _dev_ptr(gamax, torch.float32, ng),
                                       _dev_ptr(workspace, torch.float32, ACT_WORKSPACE_FLOATS),
                                       _dev_ptr(tamax, torch.float32, 1), _dev_ptr(tscale, torch.float32, 1),
                                       _dev_ptr(q, torch.uint8, n), _stream()))
    return q, tscale, gamax, tamax


def coat_act_quant_tensor_from_group_amax(x_bf16, group_amax, G: int = 16, out=None, workspace=None):
    """The same with the group maxima supplied by the caller -> (codes, tensor_scale, tensor_amax)."""
    import torch
    n = x_bf16.numel()
    ng = n_groups(n, G) if G > 0 else 0
    dev = x_bf16.device
    if out is None:
        out = (torch.empty(n, dtype=torch.uint8, device=dev), torch.empty(1, dtype=torch.float32, device=dev),
               torch.empty(1, dtype=torch.float32, device=dev))
    if workspace is None:
        workspace = act_workspace(dev)
    q, tscale, tamax = out
    _check(lib().coat_act_quant_tensor_from_group_amax(
        _dev_ptr(x_bf16, torch.bfloat16), n, G, _dev_ptr(group_amax, torch.float32, ng),
        _dev_ptr(workspace, torch.float32, ACT_WORKSPACE_FLOATS),
        _dev_ptr(tamax, torch.float32, 1), _dev_ptr(tscale, torch.float32, 1), _dev_ptr(q, torch.uint8, n), _stream()))
    return q, tscale, tamax
