"""GPU parity: newton_schulz (C-ABI) against the fp64 oracle, element by element, on seeded
inputs whose shapes span several 128/256 tiles and ragged tails."""
import numpy as np
import pytest
import torch

import paper_2505_23725_amd as mlc
import synth_inputs as S
from oracle import muon
from helpers import NS_TOL, assert_ns_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run(x_cpu: torch.Tensor, iters=5, ws_bytes=None, coeffs=muon.NS_COEFFS, inplace=False):
    cnt, m, n = (1, *x_cpu.shape) if x_cpu.dim() == 2 else x_cpu.shape
    x = x_cpu.to(DEV)
    out = x if inplace else torch.empty_like(x)
    need = mlc.newton_schulz_workspace_bytes(cnt, m, n) if ws_bytes is None else ws_bytes
    ws = torch.empty(need, dtype=torch.uint8, device=DEV)
    mlc.newton_schulz(x, out, ws, iters=iters, a=coeffs[0], b=coeffs[1], c=coeffs[2])
    torch.cuda.synchronize()
    return out.cpu()


def _check(x_cpu, out_cpu, iters=5, coeffs=muon.NS_COEFFS, tol=NS_TOL):
    xs = x_cpu if x_cpu.dim() == 3 else x_cpu[None]
    os_ = out_cpu if out_cpu.dim() == 3 else out_cpu[None]
    worst = 0.0
    for i in range(xs.shape[0]):
        ref = muon.newton_schulz(to_f64(xs[i]), iters, coeffs)
        st = assert_ns_close(to_f64(os_[i]), ref, f"matrix {i} of shape {tuple(xs[i].shape)}", tol)
        worst = max(worst, st["fro"])
    return worst


SHAPES = [
    (1, 128, 128),      # one tile
    (3, 128, 512),      # tiny-config wide
    (2, 512, 128),      # tiny-config tall
    (3, 100, 380),      # ragged wide that pads to 128 x 384: one-workgroup chain, L = 384
    (2, 128, 640),      # short side 128 but too long for the one-workgroup chain
    (2, 200, 136),      # ragged in both dimensions (pads to 256 x 256)
    (1, 72, 1000),      # ragged wide, row length not a multiple of 8? (1000 is) -> padded columns
    (1, 333, 77),       # ragged tall, odd row length: scalar load path; chain held transposed
    (300, 128, 256),    # more matrices than compute units on the one-workgroup chain
    (5, 384, 640),      # several tiles, wide
    (2, 640, 384),      # several tiles, tall
    (4, 768, 768),      # 150M-scale attention shape
]


@pytest.mark.parametrize("cnt,m,n", SHAPES)
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_newton_schulz_matches_oracle(cnt, m, n, dtype):
    x = S.normal((cnt, m, n), S.GRAD_STD, seed=0, stream=m * 131 + n, dtype=dtype)
    out = _run(x)
    worst = _check(x, out)
    print(f"NS {cnt}x{m}x{n} {dtype}: worst rel. Frobenius error {worst:.3e}")


@pytest.mark.parametrize("iters", [0, 1, 2, 7])
def test_iteration_counts(iters):
    x = S.normal((2, 256, 384), 1.0, seed=1, stream=iters, dtype=torch.bfloat16)
    out = _run(x, iters=iters)
    # iters = 0 is a pure scaling: only bf16 rounding separates it from the oracle
    _check(x, out, iters=iters, tol=4e-3 if iters == 0 else NS_TOL)


def test_cubic_coefficients_and_in_place():
    x = S.normal((2, 256, 256), 0.02, seed=2, stream=0, dtype=torch.float32)
    out = _run(x, iters=6, coeffs=(1.5, -0.5, 0.0), inplace=True)
    _check(x, out, iters=6, coeffs=(1.5, -0.5, 0.0))


def test_chunked_work_space_gives_same_result():
    x = S.normal((5, 256, 384), S.GRAD_STD, seed=3, stream=0, dtype=torch.bfloat16)
    full = _run(x)
    two = _run(x, ws_bytes=2 * mlc.newton_schulz_workspace_min_bytes(256, 384))
    one = _run(x, ws_bytes=mlc.newton_schulz_workspace_min_bytes(256, 384))
    assert torch.equal(full.view(torch.int16), two.view(torch.int16))
    assert torch.equal(full.view(torch.int16), one.view(torch.int16))


def test_zero_matrix_and_determinism():
    x = S.normal((3, 128, 256), S.GRAD_STD, seed=4, stream=0, dtype=torch.bfloat16)
    x[1].zero_()
    a = _run(x)
    b = _run(x)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    assert torch.count_nonzero(a[1]) == 0
    assert torch.isfinite(a.float()).all()
    _check(x, a)


def test_zero_matrix_with_eps_zero_stays_zero():
    # 1 / (norm + eps) must not turn into inf * 0 when both the matrix and eps are zero
    for shape in [(2, 128, 256), (2, 256, 384)]:      # one-workgroup chain, batched products
        x = S.normal(shape, S.GRAD_STD, seed=6, stream=shape[2], dtype=torch.bfloat16)
        x[0].zero_()
        xd = x.to(DEV)
        out = torch.empty_like(xd)
        ws = torch.empty(mlc.newton_schulz_workspace_bytes(*shape), dtype=torch.uint8, device=DEV)
        for iters in (0, 5):
            mlc.newton_schulz(xd, out, ws, iters=iters, eps=0.0)
            torch.cuda.synchronize()
            o = out.cpu()
            assert torch.count_nonzero(o[0]) == 0
            assert torch.isfinite(o.float()).all()
            ref = muon.newton_schulz(to_f64(x[1]), iters, eps=0.0)
            assert_ns_close(to_f64(o[1]), ref, f"{shape} eps=0 iters={iters}", 4e-3 if iters == 0 else NS_TOL)


@pytest.mark.parametrize("cnt,m,n", [(100, 256, 256), (230, 256, 256), (70, 384, 384), (45, 256, 512), (45, 512, 256)])
def test_more_small_tiles_than_compute_units(cnt, m, n):
    """Batches whose products run the 128 x 128 tile with more tiles than compute units (a CU must
    never hold two of these workgroups: the second one's tiles once came out as garbage): every
    matrix finite, two runs bit-identical, and matrices from the end of the batch, where the
    workgroups beyond the first 256 work, match the oracle."""
    x = S.normal((cnt, m, n), S.GRAD_STD, seed=8, stream=cnt + n, dtype=torch.bfloat16)
    a = _run(x)
    b = _run(x)
    assert torch.isfinite(a.float()).all()
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for i in (cnt // 8 - 1, cnt // 8, cnt - 1):       # around the end of the first XCD's range, and the last
        assert_ns_close(to_f64(a[i]), muon.newton_schulz(to_f64(x[i]), 5), f"matrix {i} of {cnt} x {m} x {n}")


def test_singular_values_land_in_the_band():
    x = S.normal((1, 256, 512), S.GRAD_STD, seed=5, stream=0, dtype=torch.bfloat16)
    out = _run(x)
    sv = np.linalg.svd(to_f64(out[0]), compute_uv=False)
    # band of the tuned quintic, widened by the bf16 error budget
    assert sv.max() <= 1.2024 * (1 + 2 * NS_TOL)
    assert np.median(sv) >= 0.6818 * (1 - 2 * NS_TOL)


def test_work_space_too_small_is_an_error():
    x = torch.zeros(1, 128, 128, dtype=torch.bfloat16, device=DEV)
    ws = torch.empty(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(mlc.MulocoError) as e:
        mlc.newton_schulz(x, x, ws)
    assert e.value.code == -4
