"""GPU parity: error feedback (Algorithm 2, EF branch) and the 2- and 8-bit forms of the
row-wise quantiser through the C-ABI, against the oracle: codes, scales and residuals bit for
bit, the outer update within the elementwise tolerances."""
import numpy as np
import pytest
import torch

import paper_2505_23725_amd as mlc
import synth_inputs as S
from oracle import diloco
from helpers import assert_fp32_close, assert_stored_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(cnt, m, n, K, wdtype, gdtype, seed):
    tg = S.normal((cnt, m, n), S.PARAM_STD, seed, 0, dtype=gdtype)
    ws = [(tg.float() - S.normal((cnt, m, n), S.DELTA_STD, seed, 10 + k)).to(wdtype) for k in range(K)]
    u = S.normal((cnt, m, n), 1e-3, seed, 5, dtype=torch.float32)
    return tg, ws, u


def _alloc(cnt, m, n, K, bits):
    codes = [torch.full((cnt * m, n * bits // 8), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(K)]
    scales = [torch.full((cnt * m,), -1.0, dtype=torch.float32, device=DEV) for _ in range(K)]
    return codes, scales


def _same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    return np.array_equal(a.view(np.uint32), b.view(np.uint32))


BIT_CASES = [
    # cnt, m, n, K, worker dtype, global dtype
    (2, 64, 128, 3, torch.bfloat16, torch.float32),
    (1, 50, 1000, 2, torch.bfloat16, torch.float32),
    (1, 9, 12, 2, torch.float32, torch.float32),          # short rows, not a multiple of 8: byte path
    (1, 12, 5120, 2, torch.bfloat16, torch.bfloat16),     # workgroup-per-row register path
    (1, 5, 24584, 1, torch.bfloat16, torch.float32),      # beyond the register kernel: two-pass path
    (1, 7, 520, 2, torch.float32, torch.bfloat16),        # dtype pair served by the two-pass path
]


@pytest.mark.parametrize("bits", [2, 8])
@pytest.mark.parametrize("cnt,m,n,K,wd,gd", BIT_CASES)
def test_other_bit_widths_bit_exact(bits, cnt, m, n, K, wd, gd):
    tg0, ws0, u0 = _inputs(cnt, m, n, K, wd, gd, seed=5 * n + K + bits)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [w.to(DEV) for w in ws0]
    codes, scales = _alloc(cnt, m, n, K, bits)
    grp = mlc.OuterGroup(ws, tg, u, codes, scales)
    hp = mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=bits)
    mlc.muloco_quantize_delta([grp], hp)
    torch.cuda.synchronize()
    assert torch.equal(tg.cpu(), tg0) and torch.equal(u.cpu(), u0)
    ref = diloco.outer_step(to_f64(tg0).reshape(-1, n), to_f64(u0).reshape(-1, n),
                            [to_f64(w).reshape(-1, n) for w in ws0], eta_out=0.9, mu=0.8, quant_bits=bits)
    for k in range(K):
        want = diloco.pack_codes(ref["q"][k], bits)
        got = codes[k].cpu().numpy()
        assert np.array_equal(got, want), f"worker {k}: {(got != want).sum()} code bytes differ"
        assert _same_bits(scales[k].cpu().numpy(), ref["scales"][k]), f"worker {k}: scales differ"
    mlc.muloco_outer_step([grp], hp)
    torch.cuda.synchronize()
    assert_fp32_close(u.cpu().reshape(-1, n), ref["u"], "outer momentum")
    assert_stored_close(tg.cpu().reshape(-1, n), ref["theta"], "global parameters")
    for k in range(K):
        assert torch.equal(ws[k].cpu(), tg.cpu().to(wd)), f"worker {k} write-back differs from theta_g"


EF_CASES = [
    # cnt, m, n, K, worker dtype, global dtype, bits, beta
    (2, 64, 128, 3, torch.bfloat16, torch.float32, 4, 1.0),
    (1, 50, 1000, 2, torch.bfloat16, torch.float32, 4, 0.9),
    (1, 9, 6, 2, torch.float32, torch.float32, 4, 0.5),               # byte path
    (1, 12, 5120, 2, torch.bfloat16, torch.bfloat16, 4, 1.0),
    (1, 6, 20480, 2, torch.bfloat16, torch.float32, 4, 0.9),          # two launches: quantise, consume
    (1, 5, 24584, 1, torch.bfloat16, torch.float32, 4, 1.0),          # two-pass quantiser
    (1, 24, 768, 4, torch.bfloat16, torch.float32, 2, 1.0),
    (1, 24, 768, 4, torch.bfloat16, torch.float32, 8, 0.75),
]


@pytest.mark.parametrize("cnt,m,n,K,wd,gd,bits,beta", EF_CASES)
def test_error_feedback_rounds_bit_exact(cnt, m, n, K, wd, gd, bits, beta):
    """Three synchronisation rounds with carried residuals.  Every round starts from the
    values the device holds (so a bf16 global copy does not let the two sides drift), and
    compares codes, scales and the new residuals bit for bit and the update within
    tolerance; the compressor alone and the full outer step must agree with each other."""
    seed = 7 * n + K + bits
    tg0, ws0, u0 = _inputs(cnt, m, n, K, wd, gd, seed)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [w.to(DEV) for w in ws0]
    res = [torch.zeros((cnt, m, n), dtype=torch.float32, device=DEV) for _ in range(K)]
    codes, scales = _alloc(cnt, m, n, K, bits)
    grp = mlc.OuterGroup(ws, tg, u, codes, scales, res)
    hp = mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=bits, error_feedback=True, ef_beta=beta)
    for rnd in range(3):
        if rnd:     # workers moved away from the (written-back) global copy again
            for k in range(K):
                step = S.normal((cnt, m, n), S.DELTA_STD, seed, 100 * rnd + k)
                ws[k].copy_((ws[k].float().cpu() - step).to(wd))
        tg_in, u_in = tg.cpu().clone(), u.cpu().clone()
        ws_in = [w.cpu().clone() for w in ws]
        res_in = [r.cpu().numpy().reshape(-1, n).copy() for r in res]
        ref = diloco.outer_step(to_f64(tg_in).reshape(-1, n), to_f64(u_in).reshape(-1, n),
                                [to_f64(w).reshape(-1, n) for w in ws_in], eta_out=0.9, mu=0.8,
                                quant_bits=bits, residuals=res_in, ef_beta=beta)
        if rnd == 1:
            # the compressor alone on copies of the residuals: same codes, scales, residuals
            res2 = [r.clone() for r in res]
            c2, s2 = _alloc(cnt, m, n, K, bits)
            mlc.muloco_quantize_delta([mlc.OuterGroup(ws, tg, u, c2, s2, res2)], hp)
            torch.cuda.synchronize()
            assert torch.equal(tg.cpu(), tg_in) and torch.equal(u.cpu(), u_in)
            for k in range(K):
                assert np.array_equal(c2[k].cpu().numpy(), diloco.pack_codes(ref["q"][k], bits))
                assert _same_bits(res2[k].cpu().numpy().reshape(-1, n), ref["residuals"][k])
        mlc.muloco_outer_step([grp], hp)
        torch.cuda.synchronize()
        for k in range(K):
            want = diloco.pack_codes(ref["q"][k], bits)
            got = codes[k].cpu().numpy()
            assert np.array_equal(got, want), f"round {rnd} worker {k}: {(got != want).sum()} code bytes differ"
            assert _same_bits(scales[k].cpu().numpy(), ref["scales"][k]), f"round {rnd} worker {k}: scales"
            assert _same_bits(res[k].cpu().numpy().reshape(-1, n), ref["residuals"][k]), \
                f"round {rnd} worker {k}: residuals differ"
        assert_fp32_close(u.cpu().reshape(-1, n), ref["u"], f"outer momentum, round {rnd}")
        assert_stored_close(tg.cpu().reshape(-1, n), ref["theta"], f"global parameters, round {rnd}")
    # residuals are in use: after three rounds they are not all zero
    assert any(torch.count_nonzero(r) > 0 for r in res)


def test_error_feedback_off_leaves_residuals_alone():
    cnt, m, n, K = 1, 16, 256, 2
    tg0, ws0, u0 = _inputs(cnt, m, n, K, torch.bfloat16, torch.float32, seed=77)
    res = [torch.full((cnt, m, n), 3.0, dtype=torch.float32, device=DEV) for _ in range(K)]
    codes, scales = _alloc(cnt, m, n, K, 4)
    grp = mlc.OuterGroup([w.to(DEV) for w in ws0], tg0.to(DEV), u0.to(DEV), codes, scales, res)
    mlc.muloco_outer_step([grp], mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=4))
    torch.cuda.synchronize()
    assert all(torch.all(r == 3.0) for r in res)
    ref = diloco.outer_step(to_f64(tg0).reshape(-1, n), to_f64(u0).reshape(-1, n),
                            [to_f64(w).reshape(-1, n) for w in ws0], eta_out=0.9, mu=0.8, quant_bits=4)
    for k in range(K):
        assert np.array_equal(codes[k].cpu().numpy(), diloco.pack_codes4(ref["q"][k]))


SQ_CASES = [
    # cnt, m, n, K, worker dtype, global dtype, bits, error feedback
    (2, 64, 128, 3, torch.bfloat16, torch.float32, 4, False),
    (1, 50, 1000, 4, torch.bfloat16, torch.float32, 4, True),
    (1, 12, 5120, 2, torch.bfloat16, torch.bfloat16, 4, False),
    (1, 6, 16384, 2, torch.bfloat16, torch.float32, 8, False),
    (1, 5, 20480, 2, torch.bfloat16, torch.float32, 4, True),         # 15B-scale row length
    (1, 3, 24576, 1, torch.bfloat16, torch.float32, 4, False),        # longest supported row
    (1, 24, 768, 8, torch.bfloat16, torch.float32, 2, True),
    (1, 9, 2048, 1, torch.float32, torch.float32, 4, False),          # K = 1: second stage is the identity
]


@pytest.mark.parametrize("cnt,m,n,K,wd,gd,bits,ef", SQ_CASES)
def test_second_quantisation_bit_exact(cnt, m, n, K, wd, gd, bits, ef):
    seed = 11 * n + K + bits
    tg0, ws0, u0 = _inputs(cnt, m, n, K, wd, gd, seed)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [w.to(DEV) for w in ws0]
    codes, scales = _alloc(cnt, m, n, K, bits)
    res0 = [S.normal((cnt, m, n), 1e-3, seed, 40 + k) for k in range(K)] if ef else None
    res = [r.to(DEV) for r in res0] if ef else None
    mcodes = torch.full((cnt * m, n * bits // 8), 0xAA, dtype=torch.uint8, device=DEV)
    mscales = torch.full((cnt * m,), -1.0, dtype=torch.float32, device=DEV)
    grp = mlc.OuterGroup(ws, tg, u, codes, scales, res, mcodes, mscales)
    hp = mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=bits, error_feedback=ef, ef_beta=0.9,
                          second_quantisation=True)
    mlc.muloco_outer_step([grp], hp)
    torch.cuda.synchronize()
    ref = diloco.outer_step(to_f64(tg0).reshape(-1, n), to_f64(u0).reshape(-1, n),
                            [to_f64(w).reshape(-1, n) for w in ws0], eta_out=0.9, mu=0.8, quant_bits=bits,
                            residuals=[r.numpy().reshape(-1, n) for r in res0] if ef else None, ef_beta=0.9,
                            second_quantisation=True)
    for k in range(K):
        assert np.array_equal(codes[k].cpu().numpy(), diloco.pack_codes(ref["q"][k], bits)), f"worker {k} codes"
        assert _same_bits(scales[k].cpu().numpy(), ref["scales"][k])
        if ef:
            assert _same_bits(res[k].cpu().numpy().reshape(-1, n), ref["residuals"][k])
    want = diloco.pack_codes(ref["mean_q"], bits)
    got = mcodes.cpu().numpy()
    assert np.array_equal(got, want), f"{(got != want).sum()} bytes of the second-stage codes differ"
    assert _same_bits(mscales.cpu().numpy(), ref["mean_scales"]), "second-stage scales differ"
    assert_fp32_close(u.cpu().reshape(-1, n), ref["u"], "outer momentum")
    assert_stored_close(tg.cpu().reshape(-1, n), ref["theta"], "global parameters")
    if K == 1 and not ef:
        assert np.array_equal(got, codes[0].cpu().numpy())
    # without buffers for the second-stage codes the update is the same
    tg2, u2 = tg0.to(DEV), u0.to(DEV)
    c2, s2 = _alloc(cnt, m, n, K, bits)
    res2 = [r.to(DEV) for r in res0] if ef else None
    mlc.muloco_outer_step([mlc.OuterGroup([w.to(DEV) for w in ws0], tg2, u2, c2, s2, res2)], hp)
    torch.cuda.synchronize()
    assert torch.equal(tg2, tg) and torch.equal(u2, u)


FORM_CASES = [
    # cnt, m, n, K, worker dtype, global dtype, bits, offset, per matrix, error feedback, second quantisation
    (2, 64, 128, 3, torch.bfloat16, torch.float32, 4, True, False, False, False),
    (1, 50, 1000, 2, torch.bfloat16, torch.float32, 4, True, False, True, False),
    (1, 9, 12, 2, torch.float32, torch.float32, 4, True, False, False, False),        # byte path
    (1, 12, 5120, 2, torch.bfloat16, torch.bfloat16, 8, True, False, False, True),
    (1, 24, 768, 4, torch.bfloat16, torch.float32, 2, True, False, True, True),
    (1, 5, 24584, 1, torch.bfloat16, torch.float32, 4, True, False, False, False),    # two-pass quantiser
    (3, 64, 128, 3, torch.bfloat16, torch.float32, 4, False, True, False, False),
    (2, 50, 1000, 2, torch.bfloat16, torch.float32, 4, True, True, True, False),
    (2, 9, 13, 2, torch.float32, torch.float32, 8, False, True, False, False),        # scalar range pass
    (2, 6, 20480, 2, torch.bfloat16, torch.float32, 4, True, True, False, False),     # two launches after the ranges
    (4, 40, 2560, 4, torch.bfloat16, torch.bfloat16, 2, False, True, True, False),
]


@pytest.mark.parametrize("cnt,m,n,K,wd,gd,bits,offset,per_matrix,ef,second", FORM_CASES)
def test_quantiser_forms_bit_exact(cnt, m, n, K, wd, gd, bits, offset, per_matrix, ef, second):
    seed = 13 * n + K + bits + 2 * offset + per_matrix
    tg0, ws0, u0 = _inputs(cnt, m, n, K, wd, gd, seed)
    if per_matrix and cnt > 1:      # matrices of different magnitude: their ranges must differ
        for k in range(K):
            ws0[k][1] = (tg0[1].float() - 8 * (tg0[1].float() - ws0[k][1].float())).to(wd)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [w.to(DEV) for w in ws0]
    ranges = cnt if per_matrix else cnt * m
    codes = [torch.full((cnt * m, n * bits // 8), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(K)]
    scales = [torch.full((ranges,), -1.0, dtype=torch.float32, device=DEV) for _ in range(K)]
    offsets = [torch.full((ranges,), -1.0, dtype=torch.float32, device=DEV) for _ in range(K)] if offset else None
    res0 = [S.normal((cnt, m, n), 1e-3, seed, 40 + k) for k in range(K)] if ef else None
    res = [r.to(DEV) for r in res0] if ef else None
    mcodes = torch.full((cnt * m, n * bits // 8), 0xAA, dtype=torch.uint8, device=DEV) if second else None
    mscales = torch.full((cnt * m,), -1.0, dtype=torch.float32, device=DEV) if second else None
    moffsets = torch.full((cnt * m,), -1.0, dtype=torch.float32, device=DEV) if second and offset else None
    grp = mlc.OuterGroup(ws, tg, u, codes, scales, res, mcodes, mscales, offsets, moffsets)
    hp = mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=bits, error_feedback=ef, ef_beta=0.9,
                          second_quantisation=second, quant_offset=offset, quant_per_matrix=per_matrix)
    ref = diloco.outer_step(to_f64(tg0).reshape(-1, n), to_f64(u0).reshape(-1, n),
                            [to_f64(w).reshape(-1, n) for w in ws0], eta_out=0.9, mu=0.8, quant_bits=bits,
                            residuals=[r.numpy().reshape(-1, n) for r in res0] if ef else None, ef_beta=0.9,
                            second_quantisation=second, quant_offset=offset,
                            quant_scope="matrix" if per_matrix else "row", rows_per_matrix=m)
    pack = diloco.pack_codes_unsigned if offset else diloco.pack_codes

    def check_compressor(codes_, scales_, offsets_, res_):
        for k in range(K):
            got, want = codes_[k].cpu().numpy(), pack(ref["q"][k], bits)
            assert np.array_equal(got, want), f"worker {k}: {(got != want).sum()} code bytes differ"
            assert _same_bits(scales_[k].cpu().numpy(), ref["scales"][k]), f"worker {k}: scales differ"
            if offset:
                assert _same_bits(offsets_[k].cpu().numpy(), ref["offsets"][k]), f"worker {k}: offsets differ"
            if ef:
                assert _same_bits(res_[k].cpu().numpy().reshape(-1, n), ref["residuals"][k]), f"worker {k}: residuals"

    if not second:      # the compressor alone, on copies of what it updates
        c2 = [c.clone() for c in codes]
        s2 = [x.clone() for x in scales]
        o2 = [x.clone() for x in offsets] if offset else None
        r2 = [r.clone() for r in res] if ef else None
        mlc.muloco_quantize_delta([mlc.OuterGroup(ws, tg, u, c2, s2, r2, None, None, o2)], hp)
        torch.cuda.synchronize()
        assert torch.equal(tg.cpu(), tg0) and torch.equal(u.cpu(), u0)
        check_compressor(c2, s2, o2, r2)
    mlc.muloco_outer_step([grp], hp)
    torch.cuda.synchronize()
    check_compressor(codes, scales, offsets, res)
    if second:
        assert np.array_equal(mcodes.cpu().numpy(), pack(ref["mean_q"], bits)), "second-stage codes differ"
        assert _same_bits(mscales.cpu().numpy(), ref["mean_scales"])
        if offset:
            assert _same_bits(moffsets.cpu().numpy(), ref["mean_offsets"])
    assert_fp32_close(u.cpu().reshape(-1, n), ref["u"], "outer momentum")
    assert_stored_close(tg.cpu().reshape(-1, n), ref["theta"], "global parameters")
    for k in range(K):
        assert torch.equal(ws[k].cpu(), tg.cpu().to(wd)), f"worker {k} write-back differs from theta_g"
