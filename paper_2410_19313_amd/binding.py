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

FLAG_EXPAND, FLAG_M_E5M2, FLAG_E5M2, FLAG_V_E5M2, FLAG_M_PLAIN, FLAG_V_PLAIN, FLAG_BF16_SCALE, FLAG_BF16_K, FLAG_PRECISE_DQ = 1, 2, 2, 4, 8, 16, 32, 64, 128
SUPPORTED_GROUP_SIZES = (32, 64, 128, 256, 512)

ACT_GROUP_SIZES = (16,) + SUPPORTED_GROUP_SIZES
ACT_WORKSPACE_FLOATS = 1024

EXPORTS = ("coat_fp8_adamw_step", "coat_fp8_adamw_step_bf16w", "coat_quant_group", "coat_dequant_group",
           "coat_act_quant_group", "coat_act_quant_tensor", "coat_act_quant_tensor_from_group_amax",
           "coat_act_quant_tensor_static", "coat_bench_copy_control", "coat_launch_shape",
           "coat_multi_plan_bytes", "coat_multi_plan_build", "coat_fp8_adamw_step_multi", "coat_shard_range",
           "coat_step_consts_compute", "coat_fp8_adamw_step_multi_consts",
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


class TensorDesc(ctypes.Structure):
    """Mirror of coat_tensor_desc."""

    _fields_ = [
        ("w", ctypes.c_void_p), ("w_bf16", ctypes.c_void_p), ("grad_bf16", ctypes.c_void_p),
        ("m_q", ctypes.c_void_p), ("m_scale", ctypes.c_void_p), ("m_k", ctypes.c_void_p),
        ("v_q", ctypes.c_void_p), ("v_scale", ctypes.c_void_p), ("v_k", ctypes.c_void_p),
        ("n", ctypes.c_uint64), ("weight_decay", ctypes.c_float), ("reserved", ctypes.c_uint32),
    ]


class StepConsts(ctypes.Structure):
    """Mirror of coat_step_consts."""

    _fields_ = [("denom_mul", ctypes.c_float), ("denom_add", ctypes.c_float), ("neg_lr", ctypes.c_double),
                ("reserved", ctypes.c_uint64 * 2)]


def step_flags(expand=True, m_e5m2=False, v_e5m2=False, m_plain=False, v_plain=False, bf16_scale=False,
               bf16_k=False, precise_dq=False) -> int:
    return ((FLAG_EXPAND if expand else 0) | (FLAG_M_E5M2 if m_e5m2 else 0) | (FLAG_V_E5M2 if v_e5m2 else 0)
            | (FLAG_M_PLAIN if m_plain else 0) | (FLAG_V_PLAIN if v_plain else 0)
            | (FLAG_BF16_SCALE if bf16_scale else 0) | (FLAG_BF16_K if bf16_k else 0)
            | (FLAG_PRECISE_DQ if precise_dq else 0))


def _scale_dtype(flags: int):
    import torch
    return torch.bfloat16 if flags & FLAG_BF16_SCALE else torch.float32


def _k_dtype(flags: int):
    import torch
    return torch.bfloat16 if flags & FLAG_BF16_K else torch.float32


def make_hparams(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1,
                 group_size=128, expand=True, k_min=0.0, k_max=0.0,
                 m_e5m2=False, v_e5m2=False, m_plain=False, v_plain=False, bf16_scale=False, bf16_k=False,
                 precise_dq=False) -> HParams:
    return HParams(lr, beta1, beta2, eps, weight_decay, int(step), int(group_size),
                   step_flags(expand, m_e5m2, v_e5m2, m_plain, v_plain, bf16_scale, bf16_k, precise_dq), k_min, k_max)


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
        L.coat_act_quant_tensor_static.restype = ctypes.c_int
        L.coat_act_quant_tensor_static.argtypes = [vp, ctypes.c_uint64, ctypes.c_int32, vp, vp, vp, vp, vp]
        L.coat_bench_copy_control.restype = ctypes.c_int
        L.coat_bench_copy_control.argtypes = [vp] * 8 + [ctypes.c_uint64, ctypes.c_int32, vp]
        L.coat_multi_plan_bytes.restype = ctypes.c_size_t
        L.coat_multi_plan_bytes.argtypes = [ctypes.POINTER(TensorDesc), ctypes.c_uint32]
        L.coat_multi_plan_build.restype = ctypes.c_int
        L.coat_multi_plan_build.argtypes = [ctypes.POINTER(TensorDesc), ctypes.c_uint32, vp, ctypes.c_size_t]
        L.coat_fp8_adamw_step_multi.restype = ctypes.c_int
        L.coat_fp8_adamw_step_multi.argtypes = [vp, vp, ctypes.POINTER(HParams), vp]
        L.coat_step_consts_compute.restype = ctypes.c_int
        L.coat_step_consts_compute.argtypes = [ctypes.POINTER(HParams), ctypes.POINTER(StepConsts)]
        L.coat_fp8_adamw_step_multi_consts.restype = ctypes.c_int
        L.coat_fp8_adamw_step_multi_consts.argtypes = [vp, vp, ctypes.POINTER(HParams), vp, vp]
        L.coat_launch_shape.restype = ctypes.c_int
        L.coat_launch_shape.argtypes = [ctypes.c_uint64, ctypes.POINTER(ctypes.c_uint32), ctypes.POINTER(ctypes.c_uint32)]
        L.coat_shard_range.restype = ctypes.c_int
        L.coat_shard_range.argtypes = [ctypes.c_uint64, ctypes.c_int32, ctypes.c_uint32, ctypes.c_uint32,
                                       ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
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
        _dev_ptr(m_q, torch.uint8, n), _dev_ptr(m_scale, _scale_dtype(hp.flags), ng), _dev_ptr(m_k, _k_dtype(hp.flags), ng),
        _dev_ptr(v_q, torch.uint8, n), _dev_ptr(v_scale, _scale_dtype(hp.flags), ng), _dev_ptr(v_k, _k_dtype(hp.flags), ng),
        n, ctypes.byref(hp), _stream()))


def coat_fp8_adamw_step_bf16w(w, w_bf16, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, hp: HParams) -> None:
    """coat_fp8_adamw_step that also writes the new weights as bfloat16 into w_bf16 [n]."""
    import torch
    n = w.numel()
    ng = n_groups(n, hp.group_size) if hp.group_size > 0 else 0
    _check(lib().coat_fp8_adamw_step_bf16w(
        _dev_ptr(w, torch.float32), _dev_ptr(w_bf16, torch.bfloat16, n), _dev_ptr(grad_bf16, torch.bfloat16, n),
        _dev_ptr(m_q, torch.uint8, n), _dev_ptr(m_scale, _scale_dtype(hp.flags), ng), _dev_ptr(m_k, _k_dtype(hp.flags), ng),
        _dev_ptr(v_q, torch.uint8, n), _dev_ptr(v_scale, _scale_dtype(hp.flags), ng), _dev_ptr(v_k, _k_dtype(hp.flags), ng),
        n, ctypes.byref(hp), _stream()))


def coat_bench_copy_control(w, grad_bf16, m_q, m_scale, m_k, v_q, v_scale, v_k, G: int) -> None:
    """The copy control of the step (same bytes, same access pattern, no arithmetic): a measurement aid.
    Destroys the buffers' contents."""
    import torch
    n = w.numel()
    ng = n_groups(n, G)
    _check(lib().coat_bench_copy_control(
        _dev_ptr(w, torch.float32), _dev_ptr(grad_bf16, torch.bfloat16, n),
        _dev_ptr(m_q, torch.uint8, n), _dev_ptr(m_scale, torch.float32, ng), _dev_ptr(m_k, torch.float32, ng),
        _dev_ptr(v_q, torch.uint8, n), _dev_ptr(v_scale, torch.float32, ng), _dev_ptr(v_k, torch.float32, ng),
        n, G, _stream()))


def coat_quant_group(x, G: int, expand: bool = True, k_min: float = 0.0, k_max: float = 0.0,
                     out=None, e5m2: bool = False, bf16_scale: bool = False, bf16_k: bool = False):
    """x fp32 [n] -> (codes uint8 [n], scale fp32 (bfloat16 with bf16_scale) [ng], k fp32 (bfloat16 with bf16_k)
    [ng]) on the device."""
    import torch
    n = x.numel()
    ng = n_groups(n, G) if G > 0 else 0
    flags = ((FLAG_EXPAND if expand else 0) | (FLAG_E5M2 if e5m2 else 0) | (FLAG_BF16_SCALE if bf16_scale else 0)
             | (FLAG_BF16_K if bf16_k else 0))
    if out is None:
        out = (torch.empty(n, dtype=torch.uint8, device=x.device),
               torch.empty(ng, dtype=_scale_dtype(flags), device=x.device),
               torch.empty(ng, dtype=_k_dtype(flags), device=x.device))
    q, scale, k = out
    _check(lib().coat_quant_group(_dev_ptr(x, torch.float32), n, G, flags,
                                  k_min, k_max, _dev_ptr(q, torch.uint8, n),
                                  _dev_ptr(scale, _scale_dtype(flags), ng), _dev_ptr(k, _k_dtype(flags), ng),
                                  _stream()))
    return q, scale, k


def coat_dequant_group(q, scale, k, G: int, out=None, e5m2: bool = False):
    """codes uint8 [n] + per-group scale (fp32 or bfloat16), k -> fp32 [n] on the device."""
    import torch
    n = q.numel()
    ng = n_groups(n, G) if G > 0 else 0
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=q.device)
    flags = ((FLAG_E5M2 if e5m2 else 0) | (FLAG_BF16_SCALE if scale.dtype == torch.bfloat16 else 0)
             | (FLAG_BF16_K if k.dtype == torch.bfloat16 else 0))
    _check(lib().coat_dequant_group(_dev_ptr(q, torch.uint8), _dev_ptr(scale, _scale_dtype(flags), ng),
                                    _dev_ptr(k, _k_dtype(flags), ng), n, G, flags,
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


def coat_act_quant_tensor_static(x_bf16, G: int, out):
    """coat_act_quant_tensor without a workspace (the library's own static device scratch) and without
    any allocation: `out` = (codes uint8 [n], tensor_scale fp32 [1], group_amax fp32 [ng], tensor_amax fp32 [1])
    must be given."""
    import torch
    n = x_bf16.numel()
    ng = n_groups(n, G) if G > 0 else 0
    q, tscale, gamax, tamax = out
    _check(lib().coat_act_quant_tensor_static(_dev_ptr(x_bf16, torch.bfloat16), n, G, _dev_ptr(gamax, torch.float32, ng),
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


def coat_shard_range(n: int, G: int, rank: int, world: int):
    """[begin, end) of the elements rank `rank` of `world` owns: contiguous, cut at multiples of G."""
    b, e = ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().coat_shard_range(n, G, rank, world, ctypes.byref(b), ctypes.byref(e)))
    return b.value, e.value


def coat_multi_plan_build(descs) -> bytes:
    """Host side of the multi-tensor step: a list of TensorDesc -> the plan blob (bytes)."""
    arr = (TensorDesc * max(1, len(descs)))(*descs)
    size = lib().coat_multi_plan_bytes(arr, len(descs))
    if size == 0:
        raise CoatError(-7, strerror(-7))
    buf = ctypes.create_string_buffer(size)
    _check(lib().coat_multi_plan_build(arr, len(descs), buf, size))
    return buf.raw


class MultiPlan:
    """The plan of a multi-tensor step: built from per-tensor device tensors, kept in host memory
    (header) and device memory (what the kernels read).  Holds references to the tensors it describes."""

    def __init__(self, tensors, G: int):
        """tensors: a list of dicts with keys w, grad, m_q, m_scale, m_k, v_q, v_scale, v_k and optionally
        w_bf16 and weight_decay (default 0.0).  G is only used to check the metadata sizes here."""
        import torch
        descs = []
        sdt = tensors[0]["m_scale"].dtype if tensors else torch.float32     # fp32, or bfloat16 for COAT_FLAG_BF16_SCALE
        self.bf16_scale = sdt == torch.bfloat16
        kdt = tensors[0]["m_k"].dtype if tensors else torch.float32         # the same for COAT_FLAG_BF16_K
        self.bf16_k = kdt == torch.bfloat16
        for t in tensors:
            n = t["w"].numel()
            ng = n_groups(n, G)
            wb = t.get("w_bf16")
            descs.append(TensorDesc(
                _dev_ptr(t["w"], torch.float32).value or 0,
                (_dev_ptr(wb, torch.bfloat16, n).value or 0) if wb is not None else 0,
                _dev_ptr(t["grad"], torch.bfloat16, n).value or 0,
                _dev_ptr(t["m_q"], torch.uint8, n).value or 0, _dev_ptr(t["m_scale"], sdt, ng).value or 0,
                _dev_ptr(t["m_k"], kdt, ng).value or 0,
                _dev_ptr(t["v_q"], torch.uint8, n).value or 0, _dev_ptr(t["v_scale"], sdt, ng).value or 0,
                _dev_ptr(t["v_k"], kdt, ng).value or 0,
                n, float(t.get("weight_decay", 0.0)), 0))
        self.tensors = list(tensors)
        self.group_size = G
        self.host = coat_multi_plan_build(descs)
        self._host_buf = ctypes.create_string_buffer(self.host, len(self.host))
        dev = tensors[0]["w"].device if tensors else torch.device("cuda")
        self.device = torch.frombuffer(bytearray(self.host), dtype=torch.uint8).to(dev)


def coat_fp8_adamw_step_multi(plan: MultiPlan, hp: HParams) -> None:
    """One fused step over every tensor of the plan in a single launch (hp.weight_decay is ignored:
    each tensor carries its own)."""
    if hp.group_size != plan.group_size:
        raise ValueError("the plan's metadata buffers were sized for G=%d" % plan.group_size)
    if bool(hp.flags & FLAG_BF16_SCALE) != plan.bf16_scale or bool(hp.flags & FLAG_BF16_K) != plan.bf16_k:
        raise ValueError("COAT_FLAG_BF16_SCALE / _K must match the dtypes of the plan's scale and k tensors")
    _check(lib().coat_fp8_adamw_step_multi(ctypes.cast(plan._host_buf, ctypes.c_void_p),
                                           ctypes.c_void_p(plan.device.data_ptr()), ctypes.byref(hp), _stream()))


def coat_step_consts_compute(hp: HParams) -> bytes:
    """The 32 bytes of step-dependent constants for hp (host side; copy them into the device block)."""
    c = StepConsts()
    _check(lib().coat_step_consts_compute(ctypes.byref(hp), ctypes.byref(c)))
    return bytes(c)


def step_consts_tensor(hp: HParams, device, out=None):
    """A device uint8[32] tensor holding coat_step_consts for hp (written into `out` when given)."""
    import torch
    host = torch.frombuffer(bytearray(coat_step_consts_compute(hp)), dtype=torch.uint8)
    if out is None:
        return host.to(device)
    out.copy_(host)
    return out


def coat_fp8_adamw_step_multi_consts(plan: MultiPlan, hp: HParams, consts) -> None:
    """coat_fp8_adamw_step_multi with the step-dependent constants read from `consts` (device uint8[32]),
    so that a captured graph can be replayed across steps."""
    import torch
    if hp.group_size != plan.group_size:
        raise ValueError("the plan's metadata buffers were sized for G=%d" % plan.group_size)
    if bool(hp.flags & FLAG_BF16_SCALE) != plan.bf16_scale or bool(hp.flags & FLAG_BF16_K) != plan.bf16_k:
        raise ValueError("COAT_FLAG_BF16_SCALE / _K must match the dtypes of the plan's scale and k tensors")
    _check(lib().coat_fp8_adamw_step_multi_consts(ctypes.cast(plan._host_buf, ctypes.c_void_p),
                                                  ctypes.c_void_p(plan.device.data_ptr()), ctypes.byref(hp),
                                                  _dev_ptr(consts, torch.uint8, ctypes.sizeof(StepConsts)), _stream()))
