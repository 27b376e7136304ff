"""CPU-only checks of the C-ABI boundary: the library loads, exports every function the
header declares, and its host-side validation rejects bad arguments before touching the
GPU (none of these calls enqueues work)."""
import ctypes as C
import os
import re

import pytest

import paper_2505_23725_amd as mlc
from paper_2505_23725_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "muloco.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b([a-z_][a-z0-9_]*)\s*\([^;{}]*\)\s*;", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = mlc.library()
    names = _declared_functions()
    assert {"newton_schulz", "muloco_inner_step", "muloco_outer_step", "muloco_quantize_delta",
            "muloco_strerror", "newton_schulz_workspace_bytes"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in muloco.h but not exported"


def test_strerror_and_codes():
    assert mlc.strerror(0) == "ok"
    for code in range(-8, 0):
        assert mlc.strerror(code) not in ("ok", "unknown error")
    assert mlc.strerror(-99) == "unknown error"


def test_workspace_sizes():
    one = mlc.newton_schulz_workspace_min_bytes(2048, 2048)
    # two X buffers + Gram + polynomial, bf16, plus small per-matrix slots
    assert one >= 4 * 2048 * 2048 * 2
    # ... and a row pitch skewed by one 128-byte line per row of each of the four buffers
    assert one < 4 * 2048 * (2048 + 64) * 2 + 16384
    assert mlc.newton_schulz_workspace_bytes(96, 2048, 2048) == 96 * one
    # padding to the 128 tile granularity
    assert mlc.newton_schulz_workspace_min_bytes(100, 130) == mlc.newton_schulz_workspace_min_bytes(128, 256)
    # tall and wide differ only by the pitch skew of their rows
    tall, wide = mlc.newton_schulz_workspace_min_bytes(512, 128), mlc.newton_schulz_workspace_min_bytes(128, 512)
    assert abs(tall - wide) == 2 * (512 - 128) * 64 * 2
    assert mlc.newton_schulz_workspace_bytes(0, 8, 8) == 0
    assert mlc.newton_schulz_workspace_min_bytes(-1, 8) == 0


def _ns(lib, inp=0x1000, out=0x1000, dtype=0, count=1, m=128, n=128, iters=5, ws=0x10000, wsb=1 << 30, eps=1e-7):
    return lib.newton_schulz(inp, out, dtype, count, m, n, iters, 3.4445, -4.775, 2.0315, eps, ws, wsb, None)


def test_static_scratch_entry_rejects_before_touching_the_gpu():
    lib = mlc.library()

    def call(inp=0x1000, out=0x1000, dtype=1, count=1, m=128, n=128, iters=5, eps=1e-7):
        return lib.newton_schulz_static_scratch(inp, out, dtype, count, m, n, iters, 3.4445, -4.775, 2.0315,
                                                eps, None)
    assert call(inp=None) == -1
    assert call(dtype=9) == -3
    assert call(count=0) == -2
    assert call(iters=-1) == -5
    assert call(out=0x1008) == -5
    # one 2048 x 8192 matrix needs more than the built-in buffer; 2048 x 2048 is the largest square
    assert mlc.newton_schulz_workspace_min_bytes(2048, 8192) > B.STATIC_SCRATCH_BYTES
    assert mlc.newton_schulz_workspace_min_bytes(2048, 2048) <= B.STATIC_SCRATCH_BYTES
    assert call(m=2048, n=8192) == -8
    assert call(m=8192, n=2048, count=3) == -8
    assert "scratch" in mlc.strerror(-8)


def test_newton_schulz_argument_errors():
    lib = mlc.library()
    assert _ns(lib, inp=None) == -1
    assert _ns(lib, out=None) == -1
    assert _ns(lib, dtype=7) == -3
    assert _ns(lib, count=0) == -2
    assert _ns(lib, m=0) == -2
    assert _ns(lib, n=-4) == -2
    assert _ns(lib, m=1 << 31) == -2
    assert _ns(lib, iters=-1) == -5
    assert _ns(lib, eps=-1.0) == -5
    assert _ns(lib, inp=0x1004) == -5                 # misaligned data pointer
    assert _ns(lib, ws=None) == -4
    assert _ns(lib, ws=0x10010) == -4                 # work space not 256-byte aligned
    assert _ns(lib, wsb=1024) == -4                   # too small for one matrix


def _inner_group(**kw):
    d = dict(count=2, m=128, n=256, param=0x1000, param_dtype=1, grad=0x2000, grad_dtype=1,
             momentum=0x3000, lr_scale=1.0)
    d.update(kw)
    return B._InnerGroup(**d)


def test_inner_step_argument_errors():
    lib = mlc.library()
    hp = B._MuonHParams(0.05, 0.01, 0.95, 1, 5, 3.4445, -4.775, 2.0315, 1e-7)

    def call(g, hp_=hp, ws=0x10000, wsb=1 << 30, n=1):
        arr = (B._InnerGroup * 1)(g)
        return lib.muloco_inner_step(arr, n, C.byref(hp_) if hp_ is not None else None, ws, wsb, None)

    assert call(_inner_group(param=None)) == -1
    assert call(_inner_group(grad=None)) == -1
    assert call(_inner_group(momentum=None)) == -1
    assert call(_inner_group(), hp_=None) == -1
    assert call(_inner_group(param_dtype=3)) == -3
    assert call(_inner_group(count=0)) == -2
    assert call(_inner_group(), wsb=100) == -4
    assert call(_inner_group(), ws=None) == -4
    assert call(_inner_group(), n=-1) == -5
    bad = B._MuonHParams(0.05, 0.01, 0.95, 1, -2, 3.4445, -4.775, 2.0315, 1e-7)
    assert call(_inner_group(), hp_=bad) == -5
    arr = (B._InnerGroup * 1)(_inner_group())
    assert lib.muloco_inner_step(arr, 0, C.byref(hp), None, 0, None) == 0     # nothing to do
    assert lib.muloco_inner_workspace_bytes(arr, 1) == 2 * mlc.newton_schulz_workspace_min_bytes(128, 256)
    assert lib.muloco_inner_workspace_min_bytes(arr, 1) == mlc.newton_schulz_workspace_min_bytes(128, 256)
    # several groups: room for all of them at once (they then share launches), not just for the largest
    arr3 = (B._InnerGroup * 3)(_inner_group(), _inner_group(), _inner_group())
    arr3[1].count, arr3[1].m, arr3[1].n = 3, 256, 256
    arr3[2].count, arr3[2].m, arr3[2].n = 1, 512, 128
    want = (arr3[0].count * mlc.newton_schulz_workspace_min_bytes(arr3[0].m, arr3[0].n)
            + 3 * mlc.newton_schulz_workspace_min_bytes(256, 256) + mlc.newton_schulz_workspace_min_bytes(512, 128))
    assert lib.muloco_inner_workspace_bytes(arr3, 3) == want
    assert lib.muloco_inner_workspace_min_bytes(arr3, 3) == max(
        mlc.newton_schulz_workspace_min_bytes(a.m, a.n) for a in arr3)


def test_outer_step_argument_errors():
    lib = mlc.library()
    K = 2
    wp = (C.c_void_p * K)(0x1000, 0x2000)
    cp = (C.c_void_p * K)(0x5000, 0x6000)
    sp = (C.c_void_p * K)(0x7000, 0x8000)

    def group(**kw):
        d = dict(count=1, m=4, n=16, worker_params=C.cast(wp, C.POINTER(C.c_void_p)), worker_dtype=1,
                 global_param=0x3000, global_dtype=0, outer_momentum=0x4000,
                 codes=C.cast(cp, C.POINTER(C.c_void_p)), scales=C.cast(sp, C.POINTER(C.c_void_p)))
        d.update(kw)
        return B._OuterGroup(**d)

    def call(g, fn="muloco_outer_step", **hpkw):
        h = dict(K=K, eta_out=0.7, mu=0.9, nesterov=1, quant_bits=0, write_back=1)
        h.update(hpkw)
        hp = B._OuterHParams(**h)
        arr = (B._OuterGroup * 1)(g)
        return getattr(lib, fn)(arr, 1, C.byref(hp), None)

    assert call(group(global_param=None)) == -1
    assert call(group(outer_momentum=None)) == -1
    assert call(group(worker_params=None)) == -1
    assert call(group(), K=0) == -5
    assert call(group(), K=33) == -5
    assert call(group(), quant_bits=3) == -5
    assert call(group(), quant_bits=16) == -5
    assert call(group(n=14), quant_bits=2) == -2      # four 2-bit codes per byte
    assert call(group(worker_dtype=9)) == -3
    assert call(group(m=0)) == -2
    assert call(group(n=15), quant_bits=4) == -2      # odd row length cannot be packed
    assert call(group(codes=None), quant_bits=4) == -1
    # error feedback needs a compressor, residual accumulators and a decay that is not negative
    assert call(group(), error_feedback=1, ef_beta=1.0) == -5
    assert call(group(), error_feedback=2, quant_bits=4, ef_beta=1.0) == -5
    assert call(group(), error_feedback=1, quant_bits=4, ef_beta=-0.5) == -5
    assert call(group(), error_feedback=1, quant_bits=4, ef_beta=1.0) == -1     # residuals NULL
    # the second quantisation needs a compressor and rows the one-pass kernel can hold
    assert call(group(), second_quantisation=1) == -5
    assert call(group(), second_quantisation=2, quant_bits=4) == -5
    assert call(group(n=24584), second_quantisation=1, quant_bits=4) == -7
    assert call(group(n=12), second_quantisation=1, quant_bits=4) == -7
    # other forms of the quantiser need a compressor; the offset form needs the offsets
    assert call(group(), quant_offset=1) == -5
    assert call(group(), quant_per_matrix=1) == -5
    assert call(group(), quant_offset=2, quant_bits=4) == -5
    assert call(group(), quant_offset=1, quant_bits=4) == -1
    assert call(group(), quant_per_matrix=1, second_quantisation=1, quant_bits=4) == -7
    null_res = (C.c_void_p * K)(0x9000, None)
    assert call(group(residuals=C.cast(null_res, C.POINTER(C.c_void_p))), error_feedback=1, quant_bits=4,
                ef_beta=1.0) == -1
    assert call(group(), fn="muloco_quantize_delta", quant_bits=0) == -5
    null_worker = (C.c_void_p * K)(0x1000, None)
    assert call(group(worker_params=C.cast(null_worker, C.POINTER(C.c_void_p)))) == -1


def test_binding_rejects_cpu_tensors_and_bad_dtypes():
    import torch
    x = torch.zeros(4, 4)
    with pytest.raises(ValueError):
        mlc.newton_schulz(x, x, torch.zeros(16, dtype=torch.uint8))
    with pytest.raises(TypeError):
        B._dtype_code(torch.zeros(2, dtype=torch.float16))


def test_adamw_argument_errors():
    lib = mlc.library()

    def call(g=None, **hpkw):
        d = dict(count=16, param=0x1000, param_dtype=0, grad=0x2000, grad_dtype=0, exp_avg=0x3000,
                 exp_avg_sq=0x4000)
        d.update(g or {})
        h = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, bias_correction=0, step=1)
        h.update(hpkw)
        arr = (B._AdamWGroup * 1)(B._AdamWGroup(**d))
        hp = B._AdamWHParams(**h)
        return lib.muloco_adamw_step(arr, 1, C.byref(hp), None)

    assert call(dict(param=None)) == -1
    assert call(dict(exp_avg_sq=None)) == -1
    assert call(dict(count=0)) == -2
    assert call(dict(grad_dtype=5)) == -3
    assert call(dict(grad=0x2004)) == -5             # misaligned
    assert call(beta1=1.0) == -5
    assert call(lr=-1.0) == -5
    assert call(bias_correction=1, step=0) == -5
    assert lib.muloco_adamw_step(None, 0, None, None) == -1


def test_topk_argument_errors():
    lib = mlc.library()
    K = 2
    wp = (C.c_void_p * K)(0x1000, 0x2000)

    def call(frac=0.1, ws=0x10000, ws_bytes=1 << 20, g=None, **hpkw):
        d = dict(count=3, m=4, n=16, worker_params=C.cast(wp, C.POINTER(C.c_void_p)), worker_dtype=1,
                 global_param=0x3000, global_dtype=0, outer_momentum=0x4000)
        d.update(g or {})
        h = dict(K=K, eta_out=0.7, mu=0.9, nesterov=1, quant_bits=0, write_back=1)
        h.update(hpkw)
        arr = (B._OuterGroup * 1)(B._OuterGroup(**d))
        hp = B._OuterHParams(**h)
        return lib.muloco_topk_outer_step(arr, 1, C.byref(hp), C.c_double(frac), ws, ws_bytes, None)

    assert call(frac=0.0) == -5 and call(frac=1.5) == -5 and call(frac=float("nan")) == -5
    assert call(quant_bits=4) == -5                       # one compressor at a time
    assert call(ws=None) == -4 and call(ws=0x10004) == -4 and call(ws_bytes=64) == -4
    assert call(error_feedback=1, ef_beta=1.0) == -1      # residuals NULL
    assert call(g=dict(global_param=None)) == -1
    arr = (B._OuterGroup * 1)(B._OuterGroup(count=3, m=4, n=16))
    assert lib.muloco_topk_workspace_bytes(arr, 1, K) == 3 * K * (2048 + 4) * 4
    assert lib.muloco_topk_workspace_bytes(arr, 1, 0) == 0
