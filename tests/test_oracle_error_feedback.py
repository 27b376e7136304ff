"""Pins for the oracle's error-feedback compressor (Sec. 2 "Compressed Communication",
Algorithm 2, EF branch) and for the 2- and 8-bit forms of the row-wise quantiser.

They fix the oracle against what the algorithm and arithmetic determine by themselves:
hand-computed rows, the conservation law of error feedback (what was not sent is kept),
the half-step bound of the residual, the classical property that components too small to
survive one quantisation are still communicated over time, and an exact-rational
definition of "nearest level"."""
from fractions import Fraction

import numpy as np

from oracle import diloco


def _rng(seed):
    return np.random.default_rng(seed)


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def test_first_round_is_the_plain_quantiser_and_the_residual_is_its_error():
    r = _rng(11)
    tg = _f32(r.standard_normal((12, 40)) * 0.02)
    tk = _f32(tg - _f32(r.standard_normal((12, 40)) * 1e-2))
    zero = np.zeros_like(tg)
    for beta in (1.0, 0.3):
        q, s, e_new = diloco.error_feedback_compress(tg, tk, zero, beta, 4)
        q0, s0 = diloco.quantize_rowwise(tg, tk, 4)
        assert np.array_equal(q, q0) and np.array_equal(s, s0)
        delta = (tg - tk).astype(np.float32)
        assert np.array_equal(e_new, (delta - diloco.dequantize_rowwise(q0, s0)).astype(np.float32))
        assert e_new.dtype == np.float32


def test_hand_rows_with_decay():
    # first synchronisation: e = 0.5 * [2,-4,0.5,0] + [6,-5,0.25,0] = [7,-7,0.5,0]; scale 1; 0.5 ties to 0
    tk = _f32([[0, 0, 0, 0]])
    E = _f32([[2, -4, 0.5, 0]])
    q, s, E1 = diloco.error_feedback_compress(_f32([[6, -5, 0.25, 0]]), tk, E, 0.5, 4)
    assert s[0] == np.float32(1) and q[0].tolist() == [7, -7, 0, 0]
    assert E1[0].tolist() == [0, 0, 0.5, 0]
    # second synchronisation: e = 0.5 * [0,0,0.5,0] + [7,0,1.25,0] = [7,0,1.5,0]; 1.5 ties to 2: more is
    # sent than was there, so the residual is negative
    q, s, E2 = diloco.error_feedback_compress(_f32([[7, 0, 1.25, 0]]), tk, E1, 0.5, 4)
    assert q[0].tolist() == [7, 0, 2, 0] and E2[0].tolist() == [0, 0, -0.5, 0]
    # beta = 0 forgets the residual: plain quantiser of the delta
    q, s, E3 = diloco.error_feedback_compress(_f32([[7, 0, 1.25, 0]]), tk, _f32([[9, 9, 9, 9]]), 0.0, 4)
    assert q[0].tolist() == [7, 0, 1, 0] and E3[0].tolist() == [0, 0, 0.25, 0]


def test_residual_stays_within_half_a_step():
    r = _rng(12)
    rows, n = 32, 64
    E = np.zeros((rows, n), np.float32)
    tg = _f32(r.standard_normal((rows, n)))
    for t in range(6):
        tk = _f32(tg - _f32(r.standard_normal((rows, n)) * 1e-2))
        q, s, E = diloco.error_feedback_compress(tg, tk, E, 0.9, 4)
        assert np.all(np.abs(E.astype(np.float64)) <= s[:, None].astype(np.float64) / 2 * (1 + 1e-6))


def test_conservation_with_beta_one():
    """sum_t sent_t + E_T = sum_t Delta_t: nothing is lost, only delayed (up to the fp32
    roundings of e and of the residual, one each per round)."""
    r = _rng(13)
    rows, n, T = 8, 48, 25
    tg = _f32(r.standard_normal((rows, n)))
    E = np.zeros((rows, n), np.float32)
    sent_sum = np.zeros((rows, n))
    delta_sum = np.zeros((rows, n))
    emax = 0.0
    for t in range(T):
        tk = _f32(tg - _f32(r.standard_normal((rows, n)) * 1e-2))
        delta_sum += (tg - tk).astype(np.float32).astype(np.float64)
        q, s, E = diloco.error_feedback_compress(tg, tk, E, 1.0, 4)
        sent_sum += diloco.dequantize_rowwise(q, s).astype(np.float64)
        emax = max(emax, float(np.max(np.abs(E))) + float(np.max(s)) * 7)
    gap = np.max(np.abs(sent_sum + E.astype(np.float64) - delta_sum))
    assert gap <= 2 * T * emax * 2.0 ** -24
    # and the gap is not zero by construction of the test: sent alone is off by the residual
    assert np.max(np.abs(sent_sum - delta_sum)) > 100 * gap


def test_small_components_are_communicated_over_time():
    """A row dominated by one entry: components below half a step never leave a plain
    quantiser; with error feedback their running sum follows the truth within one step."""
    n, T = 16, 60
    delta = np.full((1, n), 0.01, np.float32)
    delta[0, 0] = 1.0                      # step = 1/7, half a step = 0.0714 > 0.01
    tg = delta.copy()
    tk = np.zeros_like(tg)
    q, s = diloco.quantize_rowwise(tg, tk, 4)
    assert np.all(q[0, 1:] == 0)           # never sent without error feedback
    E = np.zeros_like(tg)
    sent_sum = np.zeros((1, n))
    for t in range(T):
        q, s, E = diloco.error_feedback_compress(tg, tk, E, 1.0, 4)
        sent_sum += diloco.dequantize_rowwise(q, s).astype(np.float64)
    truth = T * delta.astype(np.float64)
    assert np.all(np.abs(sent_sum - truth) <= float(s[0]) / 2 * (1 + 1e-5) + 1e-5)
    assert np.all(sent_sum[0, 1:] > 0.5 * truth[0, 1:])


def test_outer_step_with_error_feedback_averages_what_was_sent():
    r = _rng(14)
    tg = _f32(r.standard_normal((6, 16)) * 0.02).astype(np.float64)
    ths = [(_f32(tg) - _f32(r.standard_normal((6, 16)) * 1e-2)).astype(np.float64) for _ in range(3)]
    Es = [_f32(r.standard_normal((6, 16)) * 1e-3) for _ in range(3)]
    u0 = r.standard_normal((6, 16)) * 1e-3
    out = diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6, quant_bits=4, residuals=Es, ef_beta=0.9)
    sent = []
    for k in range(3):
        q, s, e_new = diloco.error_feedback_compress(_f32(tg), _f32(ths[k]), Es[k], 0.9, 4)
        assert np.array_equal(q, out["q"][k]) and np.array_equal(s, out["scales"][k])
        assert np.array_equal(e_new, out["residuals"][k])
        sent.append(diloco.dequantize_rowwise(q, s).astype(np.float64))
    psi = (sent[0] + sent[1] + sent[2]) / 3
    assert np.max(np.abs(psi - out["psi"])) < 1e-18
    u = 0.6 * u0 + 0.7 * psi
    assert np.max(np.abs(out["theta"] - (tg - 0.6 * u - 0.7 * psi))) < 1e-17
    # without residuals the plain path is taken and no residual is returned
    assert "residuals" not in diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6, quant_bits=4)


# ---- 2- and 8-bit forms --------------------------------------------------------------

def test_hand_rows_2_and_8_bit_and_packing():
    tk = _f32([[0] * 8])
    # 2 bit: levels -1, 0, 1 times amax; 0.5 ties to 0, 0.51 rounds to 1
    q, s = diloco.quantize_rowwise(_f32([[1, -1, 0.5, 0.49, -0.5, 0.51, 0, -0.75]]), tk, 2)
    assert s[0] == np.float32(1) and q[0].tolist() == [1, -1, 0, 0, 0, 1, 0, -1]
    packed = diloco.pack_codes(q, 2)
    assert packed.shape == (1, 2)
    # codes q + 2: [3,1,2,2 | 2,3,2,1], lowest column in the lowest bits
    assert packed[0, 0] == (3 | 1 << 2 | 2 << 4 | 2 << 6) and packed[0, 1] == (2 | 3 << 2 | 2 << 4 | 1 << 6)
    assert np.array_equal(diloco.unpack_codes(packed, 2), q)
    # 8 bit: amax 127 -> scale 1, integers are the levels
    q, s = diloco.quantize_rowwise(_f32([[127, -127, 0.5, 1.5, 2.5, -63.49, 100.75, 0]]), tk, 8)
    assert s[0] == np.float32(1) and q[0].tolist() == [127, -127, 0, 2, 2, -63, 101, 0]
    packed = diloco.pack_codes(q, 8)
    assert packed[0].tolist() == [255, 1, 128, 130, 130, 65, 229, 128]
    assert np.array_equal(diloco.unpack_codes(packed, 8), q)
    # the 4-bit form of the general packer is the 4-bit packer
    r = _rng(15)
    q4 = r.integers(-7, 8, size=(5, 12)).astype(np.int8)
    assert np.array_equal(diloco.pack_codes(q4, 4), diloco.pack_codes4(q4))
    assert np.array_equal(diloco.unpack_codes(diloco.pack_codes(q4, 4), 4), q4)


def test_brute_force_nearest_level_2_and_8_bit():
    r = _rng(16)
    for bits in (2, 8):
        qmax = 2 ** (bits - 1) - 1
        tg = _f32(r.standard_normal((6, 24)))
        tk = _f32(r.standard_normal((6, 24)))
        q, s = diloco.quantize_rowwise(tg, tk, bits)
        assert q.min() >= -qmax and q.max() <= qmax
        delta = (tg - tk).astype(np.float32)
        deq = diloco.dequantize_rowwise(q, s)
        assert np.all(np.abs(deq.astype(np.float64) - delta) <= s[:, None].astype(np.float64) / 2 * (1 + 1e-6))
        mism = 0
        for i in range(6):
            sc = Fraction(float(s[i]))
            for j in range(24):
                d = Fraction(float(delta[i, j]))
                k0 = int(np.floor(float(d / sc)))
                cands = [k for k in (k0 - 1, k0, k0 + 1, k0 + 2) if -qmax <= k <= qmax]
                best = min(cands, key=lambda k: (abs(d - k * sc), abs(k)))
                if best != int(q[i, j]):
                    mid = abs(abs(d / sc) - (abs(Fraction(best)) + abs(Fraction(int(q[i, j])))) / 2)
                    assert mid < Fraction(1, 2 ** 16), (bits, i, j)
                    mism += 1
        assert mism <= 2


# ---- second quantisation (dequantise - reduce - quantise between the two collectives) ----

def test_second_quantisation_of_one_worker_changes_nothing():
    """K = 1: the mean is the dequantised delta itself, and quantising dequantised values
    again reproduces them, so the second stage must be the identity."""
    r = _rng(21)
    tg = _f32(r.standard_normal((10, 32)) * 0.02).astype(np.float64)
    th = (_f32(tg) - _f32(r.standard_normal((10, 32)) * 1e-2)).astype(np.float64)
    u0 = r.standard_normal((10, 32)) * 1e-3
    for bits in (2, 4, 8):
        one = diloco.outer_step(tg, u0, [th], eta_out=0.7, mu=0.9, quant_bits=bits)
        two = diloco.outer_step(tg, u0, [th], eta_out=0.7, mu=0.9, quant_bits=bits, second_quantisation=True)
        assert np.array_equal(two["mean_q"], one["q"][0])
        assert np.all(np.abs(two["mean_scales"] - one["scales"][0]) <= np.spacing(one["scales"][0]))
        assert np.max(np.abs(two["theta"] - one["theta"])) <= 1e-9 * np.max(np.abs(one["theta"]))


def test_second_quantisation_hand_rows():
    # sent values [7, 1, -3, 0] and [7, 3, -4, 1] (scales 1): fp32 mean [7, 2, -3.5, 0.5];
    # amax 7 -> scale 1; -3.5 ties to -4, 0.5 ties to 0
    q, s, psi = diloco.requantize_mean([_f32([[7, 1, -3, 0]]), _f32([[7, 3, -4, 1]])], 4)
    assert psi[0].tolist() == [7, 2, -3.5, 0.5] and s[0] == np.float32(1)
    assert q[0].tolist() == [7, 2, -4, 0]
    # three workers: the mean is acc * fl32(1/3), not acc / 3
    a = _f32([[3, 6, -9, 21]])
    q, s, psi = diloco.requantize_mean([a, a, a], 4)
    third = np.float32(1) / np.float32(3)
    assert np.array_equal(psi, ((a + a).astype(np.float32) + a).astype(np.float32) * third)


def test_outer_step_second_stage_is_the_hand_pinned_stage():
    """The whole outer step with K = 3 must feed its update exactly what requantize_mean (pinned
    by the hand rows above, including acc * fl32(1/3)) makes of the workers' dequantised values."""
    r = _rng(23)
    tg = _f32(r.standard_normal((6, 40)) * 0.02).astype(np.float64)
    ths = [(_f32(tg) - _f32(r.standard_normal((6, 40)) * 1e-2)).astype(np.float64) for _ in range(3)]
    u0 = r.standard_normal((6, 40)) * 1e-3
    for bits in (2, 4, 8):
        two = diloco.outer_step(tg, u0, ths, eta_out=0.9, mu=0.8, quant_bits=bits, second_quantisation=True)
        sent = [diloco.dequantize_rowwise(two["q"][k], two["scales"][k]) for k in range(3)]
        q, s, _ = diloco.requantize_mean(sent, bits)
        assert np.array_equal(q, two["mean_q"])
        assert np.array_equal(s.view(np.uint32), two["mean_scales"].view(np.uint32))
        assert np.array_equal(diloco.dequantize_rowwise(q, s).astype(np.float64), two["psi"])


def test_second_quantisation_error_bound_and_use_in_the_update():
    r = _rng(22)
    tg = _f32(r.standard_normal((8, 48)) * 0.02).astype(np.float64)
    ths = [(_f32(tg) - _f32(r.standard_normal((8, 48)) * 1e-2)).astype(np.float64) for _ in range(4)]
    u0 = r.standard_normal((8, 48)) * 1e-3
    one = diloco.outer_step(tg, u0, ths, eta_out=0.9, mu=0.8, quant_bits=4)
    two = diloco.outer_step(tg, u0, ths, eta_out=0.9, mu=0.8, quant_bits=4, second_quantisation=True)
    # first-stage codes are untouched; psi moves by at most half a second-stage step
    for k in range(4):
        assert np.array_equal(one["q"][k], two["q"][k])
    half = two["mean_scales"][:, None].astype(np.float64) / 2
    assert np.all(np.abs(two["psi"] - one["psi"]) <= half * (1 + 1e-6) + 1e-9)
    assert np.max(np.abs(two["psi"] - one["psi"])) > 0
    psi = diloco.dequantize_rowwise(two["mean_q"], two["mean_scales"]).astype(np.float64)
    u = 0.8 * u0 + 0.9 * psi
    assert np.max(np.abs(two["u"] - u)) < 1e-18
    assert np.max(np.abs(two["theta"] - (tg - 0.8 * u - 0.9 * psi))) < 1e-17
