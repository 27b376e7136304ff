"""Pins for the oracle's other forms of the linear quantiser (Sec. 2 "Compressed
Communication": uniformly spaced levels over a fixed range, an offset and a number of
levels; global or row-wise): the offset form and the per-matrix scope."""
from fractions import Fraction

import numpy as np

from oracle import diloco


def _rng(seed):
    return np.random.default_rng(seed)


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def test_offset_form_hand_rows():
    v = _f32([[0, 15, 7.5, 2.5, 3.5, 14.49, 1, 8]])
    q, s, lo = diloco.quantize_values(v, 4, offset=True)
    assert s[0] == np.float32(1) and lo[0] == np.float32(0)
    assert q[0].tolist() == [0, 15, 8, 2, 4, 14, 1, 8]          # halves tie to even
    # a shift by an exactly representable amount moves the offset and nothing else
    q2, s2, lo2 = diloco.quantize_values(v - np.float32(3), 4, offset=True)
    assert np.array_equal(q2, q) and s2[0] == np.float32(1) and lo2[0] == np.float32(-3)
    deq = diloco.dequantize_values(q2, s2, lo2, offset=True)
    assert deq[0].tolist() == [-3, 12, 5, -1, 1, 11, -2, 5]
    # codes are stored unsigned: level 15 -> nibble 15, level 0 -> nibble 0
    packed = diloco.pack_codes_unsigned(q, 4)
    assert packed[0].tolist() == [0 | 15 << 4, 8 | 2 << 4, 4 | 14 << 4, 1 | 8 << 4]
    # 2 bit: three steps; 8 bit: 255 steps
    q, s, lo = diloco.quantize_values(_f32([[-1, 2, 0, 1, 0.5, -0.5, 1.5, 2]]), 2, offset=True)
    assert s[0] == np.float32(1) and lo[0] == np.float32(-1) and q[0].tolist() == [0, 3, 1, 2, 2, 0, 2, 3]
    q, s, lo = diloco.quantize_values(_f32([[0, 255, 127.5, 128.5]]), 8, offset=True)
    assert q[0].tolist() == [0, 255, 128, 128]


def test_offset_form_bounds_endpoints_and_constant_rows():
    r = _rng(31)
    v = _f32(r.standard_normal((40, 64)) * 1e-2 + 3e-3)
    v[7] = np.float32(0.125)                                   # a constant row
    for bits in (2, 4, 8):
        L = 2 ** bits - 1
        q, s, lo = diloco.quantize_values(v, bits, offset=True)
        assert q.min() >= 0 and q.max() <= L
        deq = diloco.dequantize_values(q, s, lo, offset=True)
        tol = s[:, None].astype(np.float64) / 2 * (1 + 1e-5) + 4 * np.spacing(np.abs(v).max())
        assert np.all(np.abs(deq.astype(np.float64) - v) <= tol)
        rr = np.arange(v.shape[0])
        jmin, jmax = np.argmin(v, axis=1), np.argmax(v, axis=1)
        live = s > 0
        assert np.all(q[rr, jmin][live] == 0) and np.all(q[rr, jmax][live] == L)
        assert np.array_equal(deq[rr, jmin], v[rr, jmin])      # the minimum comes back exactly
        assert s[7] == 0 and np.all(q[7] == 0) and np.all(deq[7] == np.float32(0.125))


def test_offset_form_brute_force_nearest_level():
    r = _rng(32)
    v = _f32(r.standard_normal((6, 24)))
    for bits in (2, 4):
        L = 2 ** bits - 1
        q, s, lo = diloco.quantize_values(v, bits, offset=True)
        mism = 0
        for i in range(v.shape[0]):
            sc, l0 = Fraction(float(s[i])), Fraction(float(lo[i]))
            for j in range(v.shape[1]):
                d = Fraction(float(v[i, j])) - l0
                best = min(range(L + 1), key=lambda k: (abs(d - k * sc), k))
                if best != int(q[i, j]):
                    mid = abs(d / sc - Fraction(best + int(q[i, j]), 2))
                    assert mid < Fraction(1, 2 ** 16), (bits, i, j)
                    mism += 1
        assert mism <= 2


def test_matrix_scope_is_the_row_form_of_the_flattened_matrix():
    r = _rng(33)
    m, n, cnt = 12, 16, 3
    v = _f32(r.standard_normal((cnt * m, n)) * np.repeat(np.array([1.0, 0.1, 10.0]), m)[:, None])
    for offset in (False, True):
        q, s, lo = diloco.quantize_values(v, 4, offset=offset, scope="matrix", rows_per_matrix=m)
        assert s.shape == (cnt,)
        qf, sf, lof = diloco.quantize_values(v.reshape(cnt, m * n), 4, offset=offset)
        assert np.array_equal(q.reshape(cnt, m * n), qf) and np.array_equal(s, sf) and np.array_equal(lo, lof)
        deq = diloco.dequantize_values(q, s, lo, offset=offset, scope="matrix", rows_per_matrix=m)
        deqf = diloco.dequantize_values(qf, sf, lof, offset=offset)
        assert np.array_equal(deq.reshape(cnt, m * n), deqf)
    # one range per matrix is coarser than one per row
    qr, sr, _ = diloco.quantize_values(v, 4)
    qm, sm, _ = diloco.quantize_values(v, 4, scope="matrix", rows_per_matrix=m)
    assert np.all(np.repeat(sm, m) >= sr)


def test_symmetric_row_form_of_the_general_quantiser_is_the_original_one():
    r = _rng(34)
    tg = _f32(r.standard_normal((9, 32)))
    tk = _f32(r.standard_normal((9, 32)))
    q0, s0 = diloco.quantize_rowwise(tg, tk, 4)
    q1, s1, lo1 = diloco.quantize_values((tg - tk).astype(np.float32), 4)
    assert np.array_equal(q0, q1) and np.array_equal(s0, s1) and np.all(lo1 == 0)


def test_outer_step_in_the_other_forms_averages_what_was_sent():
    r = _rng(35)
    m, n = 6, 16
    tg = _f32(r.standard_normal((2 * m, n)) * 0.02).astype(np.float64)
    ths = [(_f32(tg) - _f32(r.standard_normal((2 * m, n)) * 1e-2)).astype(np.float64) for _ in range(3)]
    u0 = r.standard_normal((2 * m, n)) * 1e-3
    for kw in (dict(quant_offset=True), dict(quant_scope="matrix", rows_per_matrix=m),
               dict(quant_offset=True, quant_scope="matrix", rows_per_matrix=m)):
        out = diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6, quant_bits=4, **kw)
        form = dict(offset=kw.get("quant_offset", False), scope=kw.get("quant_scope", "row"),
                    rows_per_matrix=kw.get("rows_per_matrix"))
        sent = [diloco.dequantize_values(out["q"][k], out["scales"][k], out["offsets"][k], **form).astype(np.float64)
                for k in range(3)]
        psi = (sent[0] + sent[1] + sent[2]) / 3
        assert np.max(np.abs(psi - out["psi"])) < 1e-18
        exact = diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6)
        groups = out["scales"][0].shape[0]
        step = np.max([out["scales"][k] for k in range(3)], axis=0)
        step = np.repeat(step, tg.shape[0] // groups)[:, None]
        assert np.all(np.abs(out["psi"] - exact["psi"]) <= step / 2 * (1 + 1e-5) + 1e-7)
