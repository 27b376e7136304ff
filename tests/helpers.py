"""Shared helpers for the GPU parity tests: conversions between torch buffers and the
float64 arrays the oracle works on, and the comparison rules.

Comparison rules (derived from the arithmetic):
* fp32 outputs of elementwise paths: relative Frobenius error <= 1e-5 per tensor.
* bf16-stored outputs of elementwise paths: each element must be a correct rounding of a
  value within 1e-5 of the oracle: |gpu - ref| <= ulp_bf16(ref)/2 + 1e-5 * max(|ref|, rms(ref)).
  The rms floor is there because these outputs are sums of terms of the tensor's typical
  magnitude (theta - mu u - eta Psi): the fp32 rounding error of such a sum scales with its
  operands, not with a result that cancellation happened to make small.
* Newton-Schulz outputs (bf16 matrix-core path): relative Frobenius error <= 2e-2 per matrix.
* quantiser codes and scales: exact equality.
"""
import numpy as np
import torch

from oracle import storage

NS_TOL = 2e-2
EW_TOL = 1e-5


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact float64 copy of what a (fp32 / bf16 / integer) tensor holds."""
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.to(torch.float32).numpy().astype(np.float64)
    return t.numpy().astype(np.float64)


def dtype_name(t: torch.Tensor) -> str:
    return {torch.float32: "f32", torch.bfloat16: "bf16"}[t.dtype]


def rel_fro(got: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    return float(num / den) if den > 0 else float(num)


def assert_fp32_close(got_t: torch.Tensor, ref: np.ndarray, what: str, tol: float = EW_TOL):
    err = rel_fro(to_f64(got_t), ref)
    assert err <= tol, f"{what}: relative Frobenius error {err:.3e} > {tol:.1e}"


def assert_bf16_rounding_of(got_t: torch.Tensor, ref: np.ndarray, what: str, tol: float = EW_TOL):
    got = to_f64(got_t)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    bound = storage.bf16_ulp(ref) * (0.5 + 2.0 ** -12) + tol * np.maximum(np.abs(ref), rms) + 1e-30
    bad = np.abs(got - ref) > bound
    assert not bad.any(), (f"{what}: {int(bad.sum())} of {bad.size} elements are not a rounding of a "
                           f"value within {tol:.0e} of the oracle; worst "
                           f"{np.max(np.abs(got - ref) / bound):.3f}x the bound")


def assert_stored_close(got_t: torch.Tensor, ref: np.ndarray, what: str):
    if got_t.dtype == torch.bfloat16:
        assert_bf16_rounding_of(got_t, ref, what)
    else:
        assert_fp32_close(got_t, ref, what)


def update_error_bf16(W_gpu_t: torch.Tensor, W0: np.ndarray, W_ref: np.ndarray) -> float:
    """Relative Frobenius error of the update when the result was stored in bf16.

    W_gpu - W_ref = (storage rounding, |.| <= ulp/2, mean square ulp^2/12, independent of the
    update) + (error of the update).  The rounding part is removed in quadrature with its
    expectation, which is far tighter than allowing half an ulp per element."""
    d = to_f64(W_gpu_t) - W_ref
    ulp = storage.bf16_ulp(W_ref)
    excess = float(np.sum(d * d) - np.sum(ulp * ulp) / 12.0)
    return float(np.sqrt(max(excess, 0.0)) / np.linalg.norm(W_ref - W0))
