"""Shared helpers for the GPU parity tests: conversions between torch buffers and the
float64 arrays the oracle works on, and the comparison rules.

Comparison rules (derived from the arithmetic):
* fp32 outputs of elementwise paths: relative Frobenius error <= 1e-5 per tensor.
* bf16-stored outputs of elementwise paths: each element must be a correct rounding of a
  value within 1e-5 of the oracle: |gpu - ref| <= ulp_bf16(ref)/2 + 1e-5 * max(|ref|, rms(ref)).
  The rms floor is there because these outputs are sums of terms of the tensor's typical
  magnitude (theta - mu u - eta Psi): the fp32 rounding error of such a sum scales with its
  operands, not with a result that cancellation happened to make small.
* Newton-Schulz outputs (bf16 matrix-core path): relative Frobenius error <= 2e-2 per matrix,
  and so that a wrong block cannot hide in the norm of a large matrix: the same ratio on
  every 256 x 256 block of the output (<= 3e-2: a block averages over fewer elements), and
  the largest element error <= 16 x the rms error and <= a quarter of the largest element
  (bf16 rounding errors scale with the element, and elements reach 5-6 x their rms, so the
  largest error of 1.7e7 elements sits near 10 x the rms error on a correct result).
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


NS_TILE = 256          # block edge of the per-block check (the GEMM's output tile)
NS_TILE_TOL = 3e-2
NS_MAX_OVER_RMS = 16.0
NS_MAX_FRACTION = 0.25


def ns_error_stats(got: np.ndarray, ref: np.ndarray) -> dict:
    """Error figures of one Newton-Schulz output against the oracle's."""
    d = got - ref
    m, n = ref.shape
    worst_tile, where = 0.0, (0, 0)
    for i in range(0, m, NS_TILE):
        for j in range(0, n, NS_TILE):
            den = np.linalg.norm(ref[i:i + NS_TILE, j:j + NS_TILE])
            num = np.linalg.norm(d[i:i + NS_TILE, j:j + NS_TILE])
            r = float(num / den) if den > 0 else float(num)
            if r > worst_tile:
                worst_tile, where = r, (i, j)
    rms = float(np.sqrt(np.mean(d * d)))
    return {"fro": rel_fro(got, ref), "tile": worst_tile, "tile_at": where,
            "max": float(np.max(np.abs(d))), "rms": rms, "ref_max": float(np.max(np.abs(ref)))}


def assert_ns_close(got: np.ndarray, ref: np.ndarray, what: str, tol: float = NS_TOL) -> dict:
    """All comparison rules of a Newton-Schulz output; `tol` scales every bound alike."""
    st = ns_error_stats(got, ref)
    k = tol / NS_TOL
    assert st["fro"] <= tol, f"{what}: relative Frobenius error {st['fro']:.3e} > {tol:.1e}"
    assert st["tile"] <= NS_TILE_TOL * k, (f"{what}: block at {st['tile_at']} has relative Frobenius "
                                           f"error {st['tile']:.3e} > {NS_TILE_TOL * k:.1e}")
    if st["rms"] > 0:
        assert st["max"] <= NS_MAX_OVER_RMS * st["rms"], (
            f"{what}: largest element error {st['max']:.3e} is {st['max'] / st['rms']:.1f}x the rms error")
    assert st["max"] <= NS_MAX_FRACTION * k * st["ref_max"] + 1e-30, (
        f"{what}: largest element error {st['max']:.3e} vs largest element {st['ref_max']:.3e}")
    return st


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


UPDATE_ELEMENT_C = 0.05


def assert_update_elements(W_gpu_t: torch.Tensor, W_ref: np.ndarray, O_ref: np.ndarray, step: float,
                           what: str) -> float:
    """Element-wise bound on the parameters after an inner step, so that a wrong block cannot
    hide in the Frobenius norm of the update: every element must be a storage rounding of a
    value whose orthogonalised term is off by at most UPDATE_ELEMENT_C * max|O| (the element
    bound of the Newton-Schulz output: 16 x its rms error of 1e-2, with rms(O) about a fifth
    of max|O|, plus margin).  step = eta * lr_scale.  Returns the worst ratio to the bound."""
    got = to_f64(W_gpu_t)
    half_ulp = storage.bf16_ulp(W_ref) * (0.5 + 2.0 ** -12) if W_gpu_t.dtype == torch.bfloat16 else 0.0
    bound = half_ulp + UPDATE_ELEMENT_C * abs(step) * float(np.max(np.abs(O_ref))) + 1e-6 * np.abs(W_ref)
    ratio = np.abs(got - W_ref) / bound
    worst = float(ratio.max())
    assert worst <= 1.0, (f"{what}: {int((ratio > 1).sum())} of {ratio.size} elements off by more than the "
                          f"element bound, worst {worst:.2f}x")
    return worst
