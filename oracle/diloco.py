"""fp64 oracle of the DiLoCo outer step with optional row-wise linear quantisation
(test infrastructure only).

Follows Sec. 4.1 eqs. 2-3 and Algorithm 1 (worker delta, average over K workers, SGD
with Nesterov momentum) and Algorithm 2's "compress parameter delta" branch.  Readings:

* theta^(t-1) in eq. 3 is the global copy before this outer step, the same tensor the
  deltas were measured against.
* The outer learning rate is folded into the momentum buffer exactly as printed:
  u <- mu u + eta_out Psi ; theta <- theta - mu u - eta_out Psi.
* The paper only says linear quantisation uses uniformly spaced levels; the workload
  description fixes row-wise, absmax scale, round-to-nearest, 4 bit.  Because codes must
  be reproducible bit for bit, this one stage is defined in IEEE fp32 arithmetic:
      delta = fl32(theta_g) - fl32(theta_k)          (one fp32 subtraction)
      amax  = max_j |delta_j| over the row, qmax = 2^(bits-1) - 1
      scale = amax / qmax                            (fp32 division)
      q_j   = clamp(rint(delta_j / scale), -qmax, qmax), ties to even; 0 if amax == 0
      code  = q_j + 2^(bits-1); two 4-bit codes per byte, even column in the low nibble
      dequantised value = float(q_j) * scale         (one fp32 multiplication)
  One quantisation per worker, before the average.  bits may be 8, 4 or 2: one, two or four
  codes per byte, the code of the lowest column in the lowest bits.
* Error feedback (Sec. 2 "Compressed Communication", Algorithm 2, EF branch): the residual
  E_k is kept in fp32 and the stage that feeds the quantiser is again fixed in fp32,
      e     = fl32(fl32(beta * E_k) + delta)         (a product, then a sum; not fused)
      (q, scale) = quantise(e) row-wise as above;  communicated value = float(q) * scale
      E_k  <- fl32(e - float(q) * scale)
  and the communicated values are averaged in place of the deltas.
* Second quantisation (Sec. 2 "Collectives": one dequantise-reduce-quantise between the
  all-to-all reduce-scatter and the all-gather): the reduced value is quantised again before
  it is used.  The stage is fixed in fp32 like the first one,
      acc   = ((s_1 + s_2) + ...) + s_K   with s_k = float(q_k) * scale_k, summed in fp32
      psi   = fl32(acc * fl32(1 / K))
      (q', scale') = quantise(psi) row-wise;  the outer update uses float(q') * scale'.
* Offset form (the paper's wording: uniformly spaced levels over a fixed range, an offset and
  a number of levels): the range is [lo, hi] = [min, max] of the values instead of
  [-amax, amax], with L = 2^bits - 1 steps,
      scale = fl32(fl32(hi - lo) / L)
      q_j   = clamp(rint(fl32(fl32(v_j - lo) / scale)), 0, L), ties to even; 0 if scale == 0
      code  = q_j (unsigned);  dequantised value = fl32(fl32(float(q_j) * scale) + lo).
* Scope: "row" takes the range over each row, "matrix" over each whole matrix (the paper's
  global variant, one range per parameter tensor); scale and lo are then stored per matrix.
* Top-k sparsification (Sec. 2 "Compressed Communication"): of each weight matrix the
  fraction f of entries with the largest magnitude is kept, the others are set to zero; each
  worker sparsifies once and the sparse tensors are averaged (an all-gather in the paper).
  Reading: the number kept is k = ceil(f * m * n), at least 1; the threshold tau is the k-th
  largest magnitude of the fp32 values and every entry with |v| >= tau is kept, so entries
  that tie with the k-th one are all kept and the result does not depend on any order.
"""
import numpy as np


def pseudogradient(theta_g, theta_k):
    """Delta_k = theta_global - theta_k  (Algorithm 1, parameter delta)."""
    return np.asarray(theta_g, np.float64) - np.asarray(theta_k, np.float64)


def average(deltas):
    """Psi = (1/K) sum_k Delta_k  (eq. 2)."""
    K = len(deltas)
    acc = np.zeros_like(np.asarray(deltas[0], np.float64))
    for d in deltas:
        acc = acc + np.asarray(d, np.float64)
    return acc / K


def outer_update(theta_g, u_prev, psi, eta_out, mu, nesterov=True):
    """eq. 3.  nesterov=False is plain SGD with momentum: theta <- theta - u."""
    theta_g = np.asarray(theta_g, np.float64)
    u = mu * np.asarray(u_prev, np.float64) + eta_out * psi
    if nesterov:
        theta = theta_g - mu * u - eta_out * psi
    else:
        theta = theta_g - u
    return theta, u


def quantize_values_rowwise(values_f32, bits=4):
    """Row-wise linear quantisation of a 2-D float32 array, in fp32 as specified above.

    Returns (q int8 [rows, n], scale float32 [rows])."""
    v = np.asarray(values_f32, dtype=np.float32)
    assert v.ndim == 2
    qmax = np.float32(2 ** (bits - 1) - 1)
    amax = np.max(np.abs(v), axis=1).astype(np.float32)
    scale = (amax / qmax).astype(np.float32)
    safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
    ratio = (v / safe[:, None]).astype(np.float32)
    q = np.clip(np.rint(ratio), -qmax, qmax)
    q = np.where(scale[:, None] > 0, q, 0.0).astype(np.int8)
    return q, scale


def _range_groups(v, scope, rows_per_matrix):
    """[groups, rows in group, n] view of a 2-D array for the chosen scope."""
    rows, n = v.shape
    if scope == "row":
        return v.reshape(rows, 1, n)
    assert scope == "matrix" and rows_per_matrix and rows % rows_per_matrix == 0
    return v.reshape(rows // rows_per_matrix, rows_per_matrix, n)


def quantize_values(values_f32, bits=4, offset=False, scope="row", rows_per_matrix=None):
    """Linear quantisation of a 2-D float32 array in any of the forms described above.

    Returns (q int16 [rows, n], scale float32 [groups], lo float32 [groups]); lo is zero for
    the symmetric form.  groups = rows for scope "row", rows / rows_per_matrix for "matrix"."""
    v = np.asarray(values_f32, dtype=np.float32)
    assert v.ndim == 2
    g = _range_groups(v, scope, rows_per_matrix)
    if not offset:
        qmax = np.float32(2 ** (bits - 1) - 1)
        amax = np.max(np.abs(g), axis=(1, 2)).astype(np.float32)
        scale = (amax / qmax).astype(np.float32)
        lo = np.zeros_like(scale)
        safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
        ratio = (g / safe[:, None, None]).astype(np.float32)
        q = np.clip(np.rint(ratio), -qmax, qmax)
    else:
        levels = np.float32(2 ** bits - 1)
        lo = np.min(g, axis=(1, 2)).astype(np.float32)
        hi = np.max(g, axis=(1, 2)).astype(np.float32)
        scale = ((hi - lo).astype(np.float32) / levels).astype(np.float32)
        safe = np.where(scale > 0, scale, np.float32(1.0)).astype(np.float32)
        shifted = (g - lo[:, None, None]).astype(np.float32)
        ratio = (shifted / safe[:, None, None]).astype(np.float32)
        q = np.clip(np.rint(ratio), 0, levels)
    q = np.where(scale[:, None, None] > 0, q, 0.0).astype(np.int16).reshape(v.shape)
    return q, scale, lo


def dequantize_values(q, scale, lo, offset=False, scope="row", rows_per_matrix=None):
    """Inverse of quantize_values, in fp32: float(q) * scale, plus lo in the offset form."""
    q = np.asarray(q)
    g = _range_groups(q.astype(np.float32), scope, rows_per_matrix)
    out = (g * np.asarray(scale, np.float32)[:, None, None]).astype(np.float32)
    if offset:
        out = (out + np.asarray(lo, np.float32)[:, None, None]).astype(np.float32)
    return out.reshape(q.shape)


def pack_codes_unsigned(q, bits):
    """Offset-form levels 0 .. 2^bits - 1 are stored as they are, packed like pack_codes."""
    return pack_codes(np.asarray(q, np.int16) - 2 ** (bits - 1), bits)


def quantize_rowwise(theta_g_f32, theta_k_f32, bits=4):
    """Row-wise linear quantisation of theta_g - theta_k (one fp32 subtraction first).

    Inputs are 2-D float32 arrays [rows, n] holding the stored values exactly.
    Returns (q int8 [rows, n], scale float32 [rows])."""
    tg = np.asarray(theta_g_f32, dtype=np.float32)
    tk = np.asarray(theta_k_f32, dtype=np.float32)
    assert tg.ndim == 2 and tg.shape == tk.shape
    return quantize_values_rowwise((tg - tk).astype(np.float32), bits)


def error_feedback_compress(theta_g_f32, theta_k_f32, residual_f32, beta, bits=4):
    """Algorithm 2, EF branch, for one worker: E <- beta E + Delta; Delta~ = C(E); E <- E - Delta~.

    Returns (q, scale, new residual float32); the communicated value is dequantize_rowwise(q, scale)."""
    tg = np.asarray(theta_g_f32, dtype=np.float32)
    tk = np.asarray(theta_k_f32, dtype=np.float32)
    E = np.asarray(residual_f32, dtype=np.float32)
    assert tg.ndim == 2 and tg.shape == tk.shape == E.shape
    delta = (tg - tk).astype(np.float32)
    e = ((np.float32(beta) * E).astype(np.float32) + delta).astype(np.float32)
    q, scale = quantize_values_rowwise(e, bits)
    sent = dequantize_rowwise(q, scale)
    return q, scale, (e - sent).astype(np.float32)


def topk_count(fraction, elems):
    """k = ceil(fraction * elems) in double precision, clamped to [1, elems]."""
    import math
    return int(min(elems, max(1, math.ceil(float(fraction) * float(elems)))))


def topk_sparsify(values_f32, fraction, rows_per_matrix):
    """Top-k by magnitude within each matrix of a 2-D float32 array [count * m, n].

    Returns (sparse float32 array, thresholds float32 [count])."""
    v = np.asarray(values_f32, dtype=np.float32)
    rows, n = v.shape
    assert rows % rows_per_matrix == 0
    g = v.reshape(rows // rows_per_matrix, rows_per_matrix * n)
    k = topk_count(fraction, g.shape[1])
    mag = np.abs(g)
    tau = np.sort(mag, axis=1)[:, g.shape[1] - k].astype(np.float32)     # k-th largest
    kept = np.where(mag >= tau[:, None], g, np.float32(0)).astype(np.float32)
    return kept.reshape(v.shape), tau


def pack_codes(q, bits):
    """Signed levels -> packed bytes: code = q + 2^(bits-1), 8 / bits codes per byte, the
    lowest column of a byte's group in its lowest bits."""
    assert bits in (2, 4, 8)
    per = 8 // bits
    q = np.asarray(q, dtype=np.int16)
    assert q.shape[-1] % per == 0
    c = (q + 2 ** (bits - 1)).astype(np.uint8)
    out = np.zeros(q.shape[:-1] + (q.shape[-1] // per,), dtype=np.uint8)
    for j in range(per):
        out |= (c[..., j::per] << (bits * j)).astype(np.uint8)
    return out


def unpack_codes(packed, bits):
    assert bits in (2, 4, 8)
    per = 8 // bits
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * per,), dtype=np.int16)
    mask = (1 << bits) - 1
    for j in range(per):
        out[..., j::per] = ((p >> (bits * j)) & mask).astype(np.int16) - 2 ** (bits - 1)
    return out.astype(np.int8)


def pack_codes4(q):
    """Signed 4-bit levels [-7, 7] -> packed bytes: code = q + 8, even column low nibble."""
    q = np.asarray(q, dtype=np.int16)
    assert q.shape[-1] % 2 == 0
    c = (q + 8).astype(np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_codes4(packed):
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.int8)
    out[..., 0::2] = (p & 0x0F).astype(np.int8) - 8
    out[..., 1::2] = (p >> 4).astype(np.int8) - 8
    return out


def dequantize_rowwise(q, scale):
    """float(q) * scale in fp32, returned as float32."""
    return (np.asarray(q, np.float32) * np.asarray(scale, np.float32)[:, None]).astype(np.float32)


def mean_fp32(sent):
    """fp32 mean of the workers' dequantised values, summed in worker order and multiplied by
    fl32(1 / K): Psi = fl32(((s_1 + s_2) + ... + s_K) * fl32(1 / K))."""
    K = len(sent)
    acc = np.asarray(sent[0]).astype(np.float32)
    for s in sent[1:]:
        acc = (acc + np.asarray(s).astype(np.float32)).astype(np.float32)
    inv_k = np.float32(1.0) / np.float32(K)
    return (acc * inv_k).astype(np.float32)


def requantize_mean(sent_f32, bits=4):
    """The dequantise-reduce-quantise step between the two collectives: fp32 mean of the
    workers' dequantised values in worker order, quantised row-wise again.

    Returns (q', scale', psi float32 before the second quantisation)."""
    psi = mean_fp32(sent_f32)
    q, scale = quantize_values_rowwise(psi, bits)
    return q, scale, psi


def outer_step(theta_g, u_prev, thetas, *, eta_out, mu, nesterov=True, quant_bits=0,
               residuals=None, ef_beta=1.0, second_quantisation=False, quant_offset=False,
               quant_scope="row", rows_per_matrix=None, topk_fraction=None):
    """One outer step on one 2-D tensor [rows, n].

    theta_g, thetas[k]: stored values (float64 holding fp32/bf16-representable numbers).
    residuals: per-worker EF accumulators E_k (float32) or None for no error feedback.
    Returns dict with theta (new global), u, psi, for the quantised path the per-worker
    levels q[k], scales[k] and (offset form) offsets[k], and with error feedback the new
    residuals."""
    theta_g = np.asarray(theta_g, np.float64)
    form = dict(offset=quant_offset, scope=quant_scope, rows_per_matrix=rows_per_matrix)
    out = {}
    deltas = []
    if quant_bits:
        out["q"], out["scales"], out["offsets"] = [], [], []
        if residuals is not None:
            out["residuals"] = []
        tg32 = theta_g.astype(np.float32)
        for k, th in enumerate(thetas):
            tk32 = np.asarray(th, np.float64).astype(np.float32)
            v = (tg32 - tk32).astype(np.float32)
            if residuals is not None:      # Algorithm 2, EF branch
                E = np.asarray(residuals[k], dtype=np.float32)
                v = ((np.float32(ef_beta) * E).astype(np.float32) + v).astype(np.float32)
            q, s, lo = quantize_values(v, quant_bits, **form)
            sent = dequantize_values(q, s, lo, **form)
            if residuals is not None:
                out["residuals"].append((v - sent).astype(np.float32))
            out["q"].append(q.astype(np.int8) if not quant_offset else q)
            out["scales"].append(s)
            out["offsets"].append(lo)
            deltas.append(sent.astype(np.float64))
    elif topk_fraction is not None:
        out["thresholds"] = []
        if residuals is not None:
            out["residuals"] = []
        tg32 = theta_g.astype(np.float32)
        for k, th in enumerate(thetas):
            tk32 = np.asarray(th, np.float64).astype(np.float32)
            v = (tg32 - tk32).astype(np.float32)
            if residuals is not None:      # Algorithm 2, EF branch
                E = np.asarray(residuals[k], dtype=np.float32)
                v = ((np.float32(ef_beta) * E).astype(np.float32) + v).astype(np.float32)
            sent, tau = topk_sparsify(v, topk_fraction, rows_per_matrix)
            if residuals is not None:
                out["residuals"].append((v - sent).astype(np.float32))
            out["thresholds"].append(tau)
            deltas.append(sent.astype(np.float64))
    else:
        assert residuals is None, "error feedback needs a compressor"
        for th in thetas:
            deltas.append(pseudogradient(theta_g, th))
    if second_quantisation:
        assert quant_bits, "the second quantisation needs a compressor"
        psi32 = mean_fp32(deltas)     # the stage requantize_mean pins by hand
        q2, s2, lo2 = quantize_values(psi32, quant_bits, **form)
        out["mean_q"], out["mean_scales"], out["mean_offsets"] = (
            q2.astype(np.int8) if not quant_offset else q2), s2, lo2
        psi = dequantize_values(q2, s2, lo2, **form).astype(np.float64)
    else:
        psi = average(deltas)
    theta, u = outer_update(theta_g, u_prev, psi, eta_out, mu, nesterov)
    out.update(theta=theta, u=u, psi=psi)
    return out


def streaming_due(t, H, J):
    """Partitioned communication (Sec. 2 "Partitioned Communication in Streaming DiLoCo"): with the
    layers split into J subsets and J | H, subset j (1 <= j <= J) is communicated at the inner
    steps t that are j * H / J modulo H.  Returns that j for inner step t >= 1, or None."""
    assert H % J == 0
    for j in range(1, J + 1):
        if (t - j * H // J) % H == 0:
            return j
    return None
