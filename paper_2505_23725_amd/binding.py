"""ctypes binding for include/muloco.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

MLC_F32, MLC_BF16 = 0, 1
MLC_MAX_WORKERS = 32
KERNEL_FAMILIES = ["ns_gemm", "momentum", "norm", "update", "outer", "quantize",
                   "dequant_outer", "convert", "adamw", "topk"]

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmuloco.so")
_lib = None


class MulocoError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class _InnerGroup(C.Structure):
    _fields_ = [("count", C.c_int64), ("m", C.c_int64), ("n", C.c_int64),
                ("param", C.c_void_p), ("param_dtype", C.c_int),
                ("grad", C.c_void_p), ("grad_dtype", C.c_int),
                ("momentum", C.c_void_p), ("lr_scale", C.c_float)]


class _MuonHParams(C.Structure):
    _fields_ = [("eta", C.c_float), ("weight_decay", C.c_float), ("beta", C.c_float),
                ("nesterov", C.c_int), ("ns_iters", C.c_int),
                ("ns_a", C.c_float), ("ns_b", C.c_float), ("ns_c", C.c_float),
                ("ns_eps", C.c_float)]


class _OuterGroup(C.Structure):
    _fields_ = [("count", C.c_int64), ("m", C.c_int64), ("n", C.c_int64),
                ("worker_params", C.POINTER(C.c_void_p)), ("worker_dtype", C.c_int),
                ("global_param", C.c_void_p), ("global_dtype", C.c_int),
                ("outer_momentum", C.c_void_p),
                ("codes", C.POINTER(C.c_void_p)), ("scales", C.POINTER(C.c_void_p)),
                ("residuals", C.POINTER(C.c_void_p)),
                ("mean_codes", C.c_void_p), ("mean_scales", C.c_void_p),
                ("offsets", C.POINTER(C.c_void_p)), ("mean_offsets", C.c_void_p)]


class _OuterHParams(C.Structure):
    _fields_ = [("K", C.c_int), ("eta_out", C.c_float), ("mu", C.c_float),
                ("nesterov", C.c_int), ("quant_bits", C.c_int), ("write_back", C.c_int),
                ("error_feedback", C.c_int), ("ef_beta", C.c_float),
                ("second_quantisation", C.c_int), ("quant_offset", C.c_int),
                ("quant_per_matrix", C.c_int)]


class _AdamWGroup(C.Structure):
    _fields_ = [("count", C.c_int64), ("param", C.c_void_p), ("param_dtype", C.c_int),
                ("grad", C.c_void_p), ("grad_dtype", C.c_int),
                ("exp_avg", C.c_void_p), ("exp_avg_sq", C.c_void_p)]


class _AdamWHParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("bias_correction", C.c_int), ("step", C.c_int)]


class _KernelTiming(C.Structure):
    _fields_ = [("launches", C.c_int64), ("total_ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


def library_path() -> str:
    return _LIB_PATH


def library() -> C.CDLL:
    """Load libmuloco.so (built in-tree by build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2505_23725_amd.build` "
            "(there is no fallback implementation)")
    lib = C.CDLL(_LIB_PATH)
    lib.muloco_strerror.restype = C.c_char_p
    lib.muloco_strerror.argtypes = [C.c_int]
    lib.newton_schulz_workspace_bytes.restype = C.c_size_t
    lib.newton_schulz_workspace_bytes.argtypes = [C.c_int64] * 3
    lib.newton_schulz_workspace_min_bytes.restype = C.c_size_t
    lib.newton_schulz_workspace_min_bytes.argtypes = [C.c_int64] * 2
    lib.newton_schulz.restype = C.c_int
    lib.newton_schulz.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64,
                                  C.c_int, C.c_float, C.c_float, C.c_float, C.c_float,
                                  C.c_void_p, C.c_size_t, C.c_void_p]
    lib.newton_schulz_static_scratch.restype = C.c_int
    lib.newton_schulz_static_scratch.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int64, C.c_int64,
                                                 C.c_int64, C.c_int, C.c_float, C.c_float, C.c_float,
                                                 C.c_float, C.c_void_p]
    for name in ("muloco_inner_workspace_bytes", "muloco_inner_workspace_min_bytes"):
        f = getattr(lib, name)
        f.restype = C.c_size_t
        f.argtypes = [C.POINTER(_InnerGroup), C.c_int]
    lib.muloco_inner_step.restype = C.c_int
    lib.muloco_inner_step.argtypes = [C.POINTER(_InnerGroup), C.c_int, C.POINTER(_MuonHParams),
                                      C.c_void_p, C.c_size_t, C.c_void_p]
    for name in ("muloco_outer_step", "muloco_quantize_delta"):
        f = getattr(lib, name)
        f.restype = C.c_int
        f.argtypes = [C.POINTER(_OuterGroup), C.c_int, C.POINTER(_OuterHParams), C.c_void_p]
    lib.muloco_topk_workspace_bytes.restype = C.c_size_t
    lib.muloco_topk_workspace_bytes.argtypes = [C.POINTER(_OuterGroup), C.c_int, C.c_int]
    lib.muloco_topk_outer_step.restype = C.c_int
    lib.muloco_topk_outer_step.argtypes = [C.POINTER(_OuterGroup), C.c_int, C.POINTER(_OuterHParams),
                                           C.c_double, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.muloco_adamw_step.restype = C.c_int
    lib.muloco_adamw_step.argtypes = [C.POINTER(_AdamWGroup), C.c_int, C.POINTER(_AdamWHParams), C.c_void_p]
    lib.muloco_timing_enable.restype = C.c_int
    lib.muloco_timing_enable.argtypes = [C.c_int]
    lib.muloco_timing_read.restype = C.c_int
    lib.muloco_timing_read.argtypes = [C.POINTER(_KernelTiming)]
    _lib = lib
    return lib


def strerror(code: int) -> str:
    return library().muloco_strerror(int(code)).decode()


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MLC_F32
    if t.dtype == torch.bfloat16:
        return MLC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}; the library takes float32 or bfloat16")


def _dev_ptr(t: torch.Tensor, what: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{what} must live on the GPU")
    if not t.is_contiguous():
        raise ValueError(f"{what} must be contiguous")
    if t.device.index != torch.cuda.current_device():
        # kernels are launched on the current device's stream; the library does no peer access
        raise ValueError(f"{what} lives on {t.device}, the current device is cuda:{torch.cuda.current_device()}")
    return t.data_ptr()


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _shape3(t: torch.Tensor):
    if t.dim() == 2:
        return 1, t.shape[0], t.shape[1]
    if t.dim() == 3:
        return tuple(t.shape)
    raise ValueError("expected a [m, n] matrix or a [count, m, n] group")


def _check(rc: int, where: str):
    if rc != 0:
        raise MulocoError(rc, where)


# ---------------------------------------------------------------------------------------
@dataclass
class MuonHParams:
    eta: float
    weight_decay: float
    beta: float = 0.9
    nesterov: bool = True
    ns_iters: int = 5
    ns_a: float = 3.4445
    ns_b: float = -4.7750
    ns_c: float = 2.0315
    ns_eps: float = 1e-7

    def _c(self) -> _MuonHParams:
        return _MuonHParams(self.eta, self.weight_decay, self.beta, int(self.nesterov),
                            int(self.ns_iters), self.ns_a, self.ns_b, self.ns_c, self.ns_eps)


@dataclass
class InnerGroup:
    """`count` same-shape matrices: param/grad/momentum are [count, m, n] (or [m, n])."""
    param: torch.Tensor
    grad: torch.Tensor
    momentum: torch.Tensor
    lr_scale: float = 1.0

    def _c(self) -> _InnerGroup:
        cnt, m, n = _shape3(self.param)
        if tuple(self.grad.shape) != tuple(self.param.shape) or \
                tuple(self.momentum.shape) != tuple(self.param.shape):
            raise ValueError("param, grad and momentum must have the same shape")
        if self.momentum.dtype != torch.float32:
            raise TypeError("momentum must be float32")
        return _InnerGroup(cnt, m, n, _dev_ptr(self.param, "param"), _dtype_code(self.param),
                           _dev_ptr(self.grad, "grad"), _dtype_code(self.grad),
                           _dev_ptr(self.momentum, "momentum"), float(self.lr_scale))


@dataclass
class OuterHParams:
    K: int
    eta_out: float
    mu: float
    nesterov: bool = True
    quant_bits: int = 0
    write_back: bool = True
    error_feedback: bool = False
    ef_beta: float = 1.0
    second_quantisation: bool = False
    quant_offset: bool = False
    quant_per_matrix: bool = False

    def _c(self) -> _OuterHParams:
        return _OuterHParams(int(self.K), self.eta_out, self.mu, int(self.nesterov),
                             int(self.quant_bits), int(self.write_back), int(self.error_feedback),
                             self.ef_beta, int(self.second_quantisation), int(self.quant_offset),
                             int(self.quant_per_matrix))


@dataclass
class OuterGroup:
    """One group of the outer step: K worker replicas, the global copy and its momentum."""
    worker_params: Sequence[torch.Tensor]
    global_param: torch.Tensor
    outer_momentum: Optional[torch.Tensor]
    codes: Optional[Sequence[torch.Tensor]] = None     # K uint8 tensors [count*m, n*bits/8]
    scales: Optional[Sequence[torch.Tensor]] = None    # K float32 tensors [count*m]
    residuals: Optional[Sequence[torch.Tensor]] = None  # K float32 tensors like the parameters
    mean_codes: Optional[torch.Tensor] = None           # uint8 [count*m, n*bits/8]: second quantisation
    mean_scales: Optional[torch.Tensor] = None          # float32 [count*m]
    offsets: Optional[Sequence[torch.Tensor]] = None    # K float32 tensors like scales (offset form)
    mean_offsets: Optional[torch.Tensor] = None         # float32 [count*m]
    _keep: list = field(default_factory=list, repr=False)

    def _c(self) -> _OuterGroup:
        cnt, m, n = _shape3(self.global_param)
        K = len(self.worker_params)
        for w in self.worker_params:
            if tuple(w.shape) != tuple(self.global_param.shape):
                raise ValueError("worker and global parameter shapes differ")
            if w.dtype != self.worker_params[0].dtype:
                raise TypeError("all workers must share one dtype")
        wp = (C.c_void_p * K)(*[_dev_ptr(w, "worker_params[k]") for w in self.worker_params])
        if self.outer_momentum is not None:
            if self.outer_momentum.dtype != torch.float32:
                raise TypeError("outer momentum must be float32")
            if self.outer_momentum.numel() != self.global_param.numel():
                raise ValueError("outer momentum shape differs")
        cp = sp = None
        if self.codes is not None:
            if self.scales is None or len(self.codes) != K:
                raise ValueError("codes need scales, K tensors each")
            for c_ in self.codes:
                if c_.dtype != torch.uint8 or c_.numel() not in [cnt * m * n * b // 8 for b in (2, 4, 8)]:
                    raise ValueError("codes[k] must be uint8 with count*m*n*bits/8 elements")
            cp = (C.c_void_p * K)(*[_dev_ptr(c_, "codes[k]") for c_ in self.codes])
        if self.scales is not None:      # quantiser scales, or the thresholds of the top-k step
            if len(self.scales) != K:
                raise ValueError("scales must hold K tensors")
            for s_ in self.scales:
                if s_.dtype != torch.float32 or s_.numel() not in (cnt * m, cnt):
                    raise ValueError("scales[k] must be float32 with count*m (or count) elements")
            sp = (C.c_void_p * K)(*[_dev_ptr(s_, "scales[k]") for s_ in self.scales])
        rp = None
        if self.residuals is not None:
            if len(self.residuals) != K:
                raise ValueError("residuals must hold K tensors")
            for r_ in self.residuals:
                if r_.dtype != torch.float32 or r_.numel() != cnt * m * n:
                    raise ValueError("residuals[k] must be float32 with count*m*n elements")
            rp = (C.c_void_p * K)(*[_dev_ptr(r_, "residuals[k]") for r_ in self.residuals])
        if self.mean_codes is not None and self.mean_codes.dtype != torch.uint8:
            raise TypeError("mean_codes must be uint8")
        if self.mean_scales is not None and (self.mean_scales.dtype != torch.float32
                                             or self.mean_scales.numel() != cnt * m):
            raise ValueError("mean_scales must be float32 with count*m elements")
        op = None
        if self.offsets is not None:
            if len(self.offsets) != K:
                raise ValueError("offsets must hold K tensors")
            for o_ in self.offsets:
                if o_.dtype != torch.float32 or o_.numel() not in (cnt * m, cnt):
                    raise ValueError("offsets[k] must be float32 with count*m (or count) elements")
            op = (C.c_void_p * K)(*[_dev_ptr(o_, "offsets[k]") for o_ in self.offsets])
        if self.mean_offsets is not None and (self.mean_offsets.dtype != torch.float32
                                              or self.mean_offsets.numel() != cnt * m):
            raise ValueError("mean_offsets must be float32 with count*m elements")
        self._keep = [wp, cp, sp, rp, op]
        return _OuterGroup(
            cnt, m, n, C.cast(wp, C.POINTER(C.c_void_p)), _dtype_code(self.worker_params[0]),
            _dev_ptr(self.global_param, "global_param"), _dtype_code(self.global_param),
            None if self.outer_momentum is None else _dev_ptr(self.outer_momentum, "outer_momentum"),
            None if cp is None else C.cast(cp, C.POINTER(C.c_void_p)),
            None if sp is None else C.cast(sp, C.POINTER(C.c_void_p)),
            None if rp is None else C.cast(rp, C.POINTER(C.c_void_p)),
            None if self.mean_codes is None else _dev_ptr(self.mean_codes, "mean_codes"),
            None if self.mean_scales is None else _dev_ptr(self.mean_scales, "mean_scales"),
            None if op is None else C.cast(op, C.POINTER(C.c_void_p)),
            None if self.mean_offsets is None else _dev_ptr(self.mean_offsets, "mean_offsets"))


# ---------------------------------------------------------------------------------------
def newton_schulz_workspace_bytes(count: int, m: int, n: int) -> int:
    return int(library().newton_schulz_workspace_bytes(count, m, n))


def newton_schulz_workspace_min_bytes(m: int, n: int) -> int:
    return int(library().newton_schulz_workspace_min_bytes(m, n))


def newton_schulz(inp: torch.Tensor, out: torch.Tensor, workspace: torch.Tensor, iters: int = 5,
                  a: float = 3.4445, b: float = -4.7750, c: float = 2.0315, eps: float = 1e-7,
                  stream=None) -> torch.Tensor:
    """out = NS_iters(inp / (||inp||_F + eps)) per matrix; `out` may be `inp`."""
    cnt, m, n = _shape3(inp)
    if tuple(out.shape) != tuple(inp.shape) or out.dtype != inp.dtype:
        raise ValueError("out must match inp in shape and dtype")
    rc = library().newton_schulz(_dev_ptr(inp, "inp"), _dev_ptr(out, "out"), _dtype_code(inp),
                                 cnt, m, n, int(iters), a, b, c, eps,
                                 _dev_ptr(workspace, "workspace"),
                                 workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "newton_schulz")
    return out


STATIC_SCRATCH_BYTES = 64 << 20


def newton_schulz_static_scratch(inp: torch.Tensor, out: torch.Tensor, iters: int = 5, a: float = 3.4445,
                                 b: float = -4.7750, c: float = 2.0315, eps: float = 1e-7,
                                 stream=None) -> torch.Tensor:
    """newton_schulz in the library's built-in scratch buffer: allocates nothing."""
    cnt, m, n = _shape3(inp)
    if tuple(out.shape) != tuple(inp.shape) or out.dtype != inp.dtype:
        raise ValueError("out must match inp in shape and dtype")
    rc = library().newton_schulz_static_scratch(_dev_ptr(inp, "inp"), _dev_ptr(out, "out"), _dtype_code(inp),
                                                cnt, m, n, int(iters), a, b, c, eps, _stream(stream))
    _check(rc, "newton_schulz_static_scratch")
    return out


def _inner_array(groups: Sequence[InnerGroup]):
    arr = (_InnerGroup * max(1, len(groups)))()
    for i, g in enumerate(groups):
        arr[i] = g._c()
    return arr


def muloco_inner_workspace_bytes(groups: Sequence[InnerGroup]) -> int:
    return int(library().muloco_inner_workspace_bytes(_inner_array(groups), len(groups)))


def muloco_inner_workspace_min_bytes(groups: Sequence[InnerGroup]) -> int:
    return int(library().muloco_inner_workspace_min_bytes(_inner_array(groups), len(groups)))


def muloco_inner_step(groups: Sequence[InnerGroup], hp: MuonHParams, workspace: torch.Tensor,
                      stream=None) -> None:
    chp = hp._c()
    rc = library().muloco_inner_step(_inner_array(groups), len(groups), C.byref(chp),
                                     _dev_ptr(workspace, "workspace"),
                                     workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "muloco_inner_step")


def _outer_array(groups: Sequence[OuterGroup]):
    arr = (_OuterGroup * max(1, len(groups)))()
    for i, g in enumerate(groups):
        arr[i] = g._c()
    return arr


def _check_outer_groups(groups: Sequence[OuterGroup], hp: OuterHParams) -> None:
    for g in groups:
        if len(g.worker_params) != hp.K:
            raise ValueError("every group needs K worker tensors")
        if hp.quant_bits in (2, 4, 8) and g.codes is not None:
            want = g.global_param.numel() * hp.quant_bits // 8
            if any(c_.numel() != want for c_ in g.codes):
                raise ValueError("codes[k] must hold count*m*n*quant_bits/8 bytes")
            if g.mean_codes is not None and g.mean_codes.numel() != want:
                raise ValueError("mean_codes must hold count*m*n*quant_bits/8 bytes")
            cnt_, m_, _ = _shape3(g.global_param)
            ranges = cnt_ if hp.quant_per_matrix else cnt_ * m_
            for t_ in list(g.scales or []) + list(g.offsets or []):
                if t_.numel() != ranges:
                    raise ValueError("scales[k] / offsets[k] must hold one entry per range")


def muloco_outer_step(groups: Sequence[OuterGroup], hp: OuterHParams, stream=None) -> None:
    _check_outer_groups(groups, hp)
    chp = hp._c()
    rc = library().muloco_outer_step(_outer_array(groups), len(groups), C.byref(chp), _stream(stream))
    _check(rc, "muloco_outer_step")


def muloco_quantize_delta(groups: Sequence[OuterGroup], hp: OuterHParams, stream=None) -> None:
    _check_outer_groups(groups, hp)
    chp = hp._c()
    rc = library().muloco_quantize_delta(_outer_array(groups), len(groups), C.byref(chp),
                                         _stream(stream))
    _check(rc, "muloco_quantize_delta")


def muloco_topk_workspace_bytes(groups: Sequence[OuterGroup], K: int) -> int:
    return int(library().muloco_topk_workspace_bytes(_outer_array(groups), len(groups), int(K)))


def muloco_topk_outer_step(groups: Sequence[OuterGroup], hp: OuterHParams, fraction: float,
                           workspace: torch.Tensor, stream=None) -> None:
    """Outer step on top-k sparsified pseudogradients; group.scales (K tensors of `count`
    floats), if given, receive the thresholds."""
    for g in groups:
        if len(g.worker_params) != hp.K:
            raise ValueError("every group needs K worker tensors")
    if workspace.dtype != torch.uint8:
        raise TypeError("workspace must be a uint8 tensor")
    chp = hp._c()
    rc = library().muloco_topk_outer_step(_outer_array(groups), len(groups), C.byref(chp), float(fraction),
                                          _dev_ptr(workspace, "workspace"), workspace.numel(), _stream(stream))
    _check(rc, "muloco_topk_outer_step")


@dataclass
class AdamWHParams:
    lr: float
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.0
    bias_correction: bool = False
    step: int = 1


def muloco_adamw_step(tensors: Sequence[tuple], hp: AdamWHParams, stream=None) -> None:
    """tensors: (param, grad, exp_avg, exp_avg_sq) tuples of equally sized device tensors."""
    arr = (_AdamWGroup * max(1, len(tensors)))()
    for i, (p_, g_, m_, v_) in enumerate(tensors):
        n = p_.numel()
        if g_.numel() != n or m_.numel() != n or v_.numel() != n:
            raise ValueError("param, grad, exp_avg and exp_avg_sq must have the same size")
        if m_.dtype != torch.float32 or v_.dtype != torch.float32:
            raise TypeError("exp_avg and exp_avg_sq must be float32")
        arr[i] = _AdamWGroup(n, _dev_ptr(p_, "param"), _dtype_code(p_), _dev_ptr(g_, "grad"), _dtype_code(g_),
                             _dev_ptr(m_, "exp_avg"), _dev_ptr(v_, "exp_avg_sq"))
    chp = _AdamWHParams(hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, int(hp.bias_correction), int(hp.step))
    rc = library().muloco_adamw_step(arr, len(tensors), C.byref(chp), _stream(stream))
    _check(rc, "muloco_adamw_step")


def muloco_timing_enable(on: bool) -> None:
    _check(library().muloco_timing_enable(int(bool(on))), "muloco_timing_enable")


def muloco_timing_read() -> dict:
    arr = (_KernelTiming * len(KERNEL_FAMILIES))()
    _check(library().muloco_timing_read(arr), "muloco_timing_read")
    return {name: {"launches": int(arr[i].launches), "total_ms": float(arr[i].total_ms),
                   "flops": float(arr[i].flops), "bytes": float(arr[i].bytes)}
            for i, name in enumerate(KERNEL_FAMILIES)}
