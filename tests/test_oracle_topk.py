"""Pins for the oracle's top-k sparsifier (Sec. 2 "Compressed Communication")."""
import numpy as np

from oracle import diloco


def _f32(x):
    return np.asarray(x, dtype=np.float32)


def test_hand_example_with_ties_and_counts():
    v = _f32([[1, -5, 3, 0.5], [2, -3, 0, 4]])            # one 2 x 4 matrix
    # a quarter of 8 entries: k = 2 -> the two largest magnitudes are 5 and 4
    s, tau = diloco.topk_sparsify(v, 0.25, rows_per_matrix=2)
    assert tau.tolist() == [4.0] and s.tolist() == [[0, -5, 0, 0], [0, 0, 0, 4]]
    # k = 3: the third largest magnitude is 3, which occurs twice: both are kept
    s, tau = diloco.topk_sparsify(v, 3 / 8, rows_per_matrix=2)
    assert tau.tolist() == [3.0] and s.tolist() == [[0, -5, 3, 0], [0, -3, 0, 4]]
    # as two 1 x 4 matrices each keeps its own top half
    s, tau = diloco.topk_sparsify(v, 0.5, rows_per_matrix=1)
    assert tau.tolist() == [3.0, 3.0] and s.tolist() == [[0, -5, 3, 0], [0, -3, 0, 4]]
    # everything, and the smallest possible fraction
    s, tau = diloco.topk_sparsify(v, 1.0, rows_per_matrix=2)
    assert np.array_equal(s, v) and tau.tolist() == [0.0]
    s, tau = diloco.topk_sparsify(v, 1e-9, rows_per_matrix=2)
    assert np.count_nonzero(s) == 1 and s[0, 1] == -5
    assert diloco.topk_count(0.005, 1000) == 5 and diloco.topk_count(0.0051, 1000) == 6
    assert diloco.topk_count(0.5, 3) == 2 and diloco.topk_count(2.0, 3) == 3


def test_against_brute_force_selection():
    r = np.random.default_rng(41)
    for frac in (0.005, 0.05, 0.2, 0.5):
        v = _f32(r.standard_normal((3 * 20, 50)))
        s, tau = diloco.topk_sparsify(v, frac, rows_per_matrix=20)
        for b in range(3):
            blk, kept = v[20 * b:20 * b + 20].ravel(), s[20 * b:20 * b + 20].ravel()
            k = diloco.topk_count(frac, blk.size)
            order = sorted(range(blk.size), key=lambda i: -abs(float(blk[i])))
            assert np.count_nonzero(kept) == k                   # continuous draws: no ties
            assert set(np.nonzero(kept)[0]) == set(order[:k])
            assert np.array_equal(kept[order[:k]], blk[order[:k]])
            assert tau[b] == abs(blk[order[k - 1]])


def test_error_feedback_with_topk_keeps_exactly_what_was_not_sent():
    r = np.random.default_rng(42)
    m, n, T = 8, 32, 12
    tg = _f32(r.standard_normal((m, n))).astype(np.float64)
    E = [np.zeros((m, n), np.float32)]
    sent_sum, delta_sum = np.zeros((m, n)), np.zeros((m, n))
    u = np.zeros((m, n))
    for t in range(T):
        th = (_f32(tg) - _f32(r.standard_normal((m, n)) * 1e-2)).astype(np.float64)
        out = diloco.outer_step(tg, u, [th], eta_out=0.0, mu=0.0, topk_fraction=0.1, rows_per_matrix=m,
                                residuals=E, ef_beta=1.0)
        delta_sum += (_f32(tg) - _f32(th)).astype(np.float64)
        sent_sum += out["psi"]
        # an entry is either sent whole (residual 0) or kept whole (nothing sent)
        assert np.all((out["psi"] == 0) | (out["residuals"][0] == 0))
        assert np.count_nonzero(out["psi"]) == diloco.topk_count(0.1, m * n)
        E = out["residuals"]
    gap = np.max(np.abs(sent_sum + E[0].astype(np.float64) - delta_sum))
    assert gap <= T * 2.0 ** -24 * np.max(np.abs(delta_sum)) * 4
    # without error feedback the small entries are simply lost
    assert np.max(np.abs(sent_sum - delta_sum)) > 1000 * gap


def test_outer_step_with_topk_averages_the_sparse_tensors():
    r = np.random.default_rng(43)
    m, n = 6, 16
    tg = _f32(r.standard_normal((2 * m, n)) * 0.02).astype(np.float64)
    ths = [(_f32(tg) - _f32(r.standard_normal((2 * m, n)) * 1e-2)).astype(np.float64) for _ in range(3)]
    u0 = r.standard_normal((2 * m, n)) * 1e-3
    out = diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6, topk_fraction=0.25, rows_per_matrix=m)
    sp = [diloco.topk_sparsify((_f32(tg) - _f32(th)).astype(np.float32), 0.25, m)[0].astype(np.float64) for th in ths]
    psi = (sp[0] + sp[1] + sp[2]) / 3
    assert np.max(np.abs(psi - out["psi"])) < 1e-18
    uu = 0.6 * u0 + 0.7 * psi
    assert np.max(np.abs(out["theta"] - (tg - 0.6 * uu - 0.7 * psi))) < 1e-17
    full = diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6, topk_fraction=1.0, rows_per_matrix=m)
    exact = diloco.outer_step(tg, u0, ths, eta_out=0.7, mu=0.6)
    assert np.max(np.abs(full["theta"] - exact["theta"])) < 1e-9
