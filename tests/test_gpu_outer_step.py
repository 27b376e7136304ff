"""GPU parity: muloco_outer_step / muloco_quantize_delta (C-ABI) against the fp64 oracle
(fp32 for the quantiser stage), element by element; codes and scales bit for bit."""
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


def _alloc_codes(cnt, m, n, K):
    codes = [torch.full((cnt * m, n // 2), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(K)]
    scales = [torch.full((cnt * m,), -1.0, dtype=torch.float32, device=DEV) for _ in range(K)]
    return codes, scales


CASES = [
    # cnt, m, n, K, worker dtype, global dtype
    (2, 128, 128, 1, torch.float32, torch.float32),
    (3, 96, 200, 8, torch.bfloat16, torch.float32),
    (1, 33, 130, 4, torch.bfloat16, torch.bfloat16),
    (1, 7, 6, 3, torch.float32, torch.float32),          # fewer than one vector per row
    (1, 5, 5, 2, torch.bfloat16, torch.float32),          # ragged tail of the flat range
    (2, 256, 768, 4, torch.bfloat16, torch.float32),
]


@pytest.mark.parametrize("cnt,m,n,K,wd,gd", CASES)
@pytest.mark.parametrize("nesterov,write_back", [(True, True), (False, False)])
def test_outer_step_matches_oracle(cnt, m, n, K, wd, gd, nesterov, write_back):
    tg0, ws0, u0 = _inputs(cnt, m, n, K, wd, gd, seed=n + K)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [w.to(DEV) for w in ws0]
    hp = mlc.OuterHParams(K=K, eta_out=0.7, mu=0.9, nesterov=nesterov, write_back=write_back)
    mlc.muloco_outer_step([mlc.OuterGroup(ws, tg, u)], hp)
    torch.cuda.synchronize()
    ref = diloco.outer_step(to_f64(tg0).reshape(-1, n), to_f64(u0).reshape(-1, n),
                            [to_f64(w).reshape(-1, n) for w in ws0], eta_out=0.7, mu=0.9,
                            nesterov=nesterov)
    assert_fp32_close(u.cpu().reshape(-1, n), ref["u"], "outer momentum")
    assert_stored_close(tg.cpu().reshape(-1, n), ref["theta"], "global parameters")
    for k in range(K):
        if write_back:
            assert_stored_close(ws[k].cpu().reshape(-1, n), ref["theta"], f"worker {k} write-back")
        else:
            assert torch.equal(ws[k].cpu(), ws0[k]), "workers must stay untouched without write-back"


QCASES = [
    (2, 64, 128, 4, torch.bfloat16, torch.float32),
    (1, 50, 1000, 2, torch.bfloat16, torch.float32),
    (1, 9, 6, 3, torch.float32, torch.float32),           # short rows: scalar path
    (1, 40, 2560, 4, torch.bfloat16, torch.bfloat16),     # a 3.1B-scale row length
    (1, 16, 10240, 1, torch.bfloat16, torch.float32),
    (1, 12, 10240, 4, torch.bfloat16, torch.float32),     # six vectors per thread, K = 4
    (1, 6, 16384, 2, torch.bfloat16, torch.float32),      # eight vectors per thread
    (1, 6, 20480, 2, torch.bfloat16, torch.float32),      # 15B-scale row length
    (1, 10, 5120, 3, torch.bfloat16, torch.float32),
    (2, 9, 2048, 2, torch.float32, torch.float32),        # widest wavefront-per-row case
    (1, 5, 24584, 1, torch.bfloat16, torch.float32),      # beyond the register kernel: two-pass path
    (1, 7, 520, 2, torch.float32, torch.bfloat16),        # dtype pair served by the two-pass path
]


@pytest.mark.parametrize("cnt,m,n,K,wd,gd", QCASES)
def test_quantised_outer_step_codes_bit_exact(cnt, m, n, K, wd, gd):
    tg0, ws0, u0 = _inputs(cnt, m, n, K, wd, gd, seed=3 * n + K)
    ws0[0][0, 1].copy_(tg0[0, 1].to(wd))                 # an all-zero delta row (if dtypes agree)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [w.to(DEV) for w in ws0]
    codes, scales = _alloc_codes(cnt, m, n, K)
    grp = mlc.OuterGroup(ws, tg, u, codes, scales)
    hp = mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=4)
    # the compressor alone first: nothing but codes and scales may change
    mlc.muloco_quantize_delta([grp], hp)
    torch.cuda.synchronize()
    assert torch.equal(tg.cpu(), tg0) and torch.equal(u.cpu(), u0)
    ref = diloco.outer_step(to_f64(tg0).reshape(-1, n), to_f64(u0).reshape(-1, n),
                            [to_f64(w).reshape(-1, n) for w in ws0], eta_out=0.9, mu=0.8, quant_bits=4)
    for k in range(K):
        want = diloco.pack_codes4(ref["q"][k])
        got = codes[k].cpu().numpy()
        assert np.array_equal(got, want), f"worker {k}: {(got != want).sum()} code bytes differ"
        assert np.array_equal(scales[k].cpu().numpy().view(np.uint32), ref["scales"][k].view(np.uint32)), \
            f"worker {k}: scales differ"
    if wd == gd or gd == torch.float32:
        zero_row = ref["scales"][0][1] == 0
        if zero_row:
            assert np.all(codes[0].cpu().numpy()[1] == 0x88)
    # the full quantised outer step (recomputes the same codes, then consumes them)
    mlc.muloco_outer_step([grp], hp)
    torch.cuda.synchronize()
    assert_fp32_close(u.cpu().reshape(-1, n), ref["u"], "outer momentum (quantised)")
    assert_stored_close(tg.cpu().reshape(-1, n), ref["theta"], "global parameters (quantised)")
    for k in range(K):   # theta_k <- theta_g: exactly what the global buffer now holds
        assert torch.equal(ws[k].cpu(), tg.cpu().to(wd)), f"worker {k} write-back differs from theta_g"
        if not (wd == torch.float32 and gd == torch.bfloat16):
            assert_stored_close(ws[k].cpu().reshape(-1, n), ref["theta"], f"worker {k} write-back")


def test_streaming_fragments_equal_one_call():
    """Calling the outer step once per fragment (a subset of groups) gives the same bits as
    one call over all groups."""
    K = 2
    hp = mlc.OuterHParams(K=K, eta_out=0.7, mu=0.9)
    groups_a, groups_b = [], []
    for i, (c, m, n) in enumerate([(2, 128, 128), (1, 128, 512), (1, 512, 128)]):
        tg0, ws0, u0 = _inputs(c, m, n, K, torch.bfloat16, torch.float32, seed=40 + i)
        for dst in (groups_a, groups_b):
            dst.append(mlc.OuterGroup([w.to(DEV) for w in ws0], tg0.to(DEV), u0.to(DEV)))
    mlc.muloco_outer_step(groups_a, hp)
    for g in groups_b:
        mlc.muloco_outer_step([g], hp)
    torch.cuda.synchronize()
    for ga, gb in zip(groups_a, groups_b):
        assert torch.equal(ga.global_param, gb.global_param)
        assert torch.equal(ga.outer_momentum, gb.outer_momentum)
        assert all(torch.equal(x, y) for x, y in zip(ga.worker_params, gb.worker_params))


def test_special_cases_on_gpu():
    # zero inner steps: identity; eta_out = 1, mu = 0: plain averaging
    K, shape = 3, (1, 64, 64)
    tg0 = S.normal(shape, S.PARAM_STD, 9, 0)
    u0 = torch.zeros(shape)
    tg, u = tg0.to(DEV), u0.to(DEV)
    ws = [tg0.clone().to(DEV) for _ in range(K)]
    mlc.muloco_outer_step([mlc.OuterGroup(ws, tg, u)], mlc.OuterHParams(K=K, eta_out=0.7, mu=0.9))
    torch.cuda.synchronize()
    assert torch.equal(tg.cpu(), tg0) and torch.count_nonzero(u) == 0
    ws0 = [tg0 - S.normal(shape, S.DELTA_STD, 9, 20 + k) for k in range(K)]
    ws = [w.to(DEV) for w in ws0]
    u = S.normal(shape, 1.0, 9, 6).to(DEV)
    mlc.muloco_outer_step([mlc.OuterGroup(ws, tg, u)], mlc.OuterHParams(K=K, eta_out=1.0, mu=0.0, write_back=False))
    torch.cuda.synchronize()
    mean = np.mean([to_f64(w) for w in ws0], axis=0)
    assert_fp32_close(tg.cpu(), mean, "plain averaging")


@pytest.mark.parametrize("quant_bits,ef", [(0, False), (4, False), (4, True), (8, False), (2, True)])
@pytest.mark.parametrize("K", [2, 8, 9])
def test_several_groups_in_one_call_equal_one_call_per_group(quant_bits, ef, K):
    """A call with several groups takes them in one launch (up to 4 groups, 8 workers; K = 9
    falls back to a launch per group).  Every output must carry the bits that a call per group
    gives: row lengths cover the wavefront-per-row and the workgroup-per-row kernels, ragged
    row counts, and for the un-quantised step a ragged flat tail."""
    shapes = [(3, 50, 256), (1, 70, 4096), (2, 33, 1000 if quant_bits else 130), (1, 5, 2048), (1, 9, 6152),
              (1, 3, 10240)]      # the last one is too long a row to share a quantised launch
    hp = mlc.OuterHParams(K=K, eta_out=0.9, mu=0.8, quant_bits=quant_bits, error_feedback=ef, ef_beta=0.9)

    def build():
        groups = []
        for gi, (cnt, m, n) in enumerate(shapes):
            tg0, ws0, u0 = _inputs(cnt, m, n, K, torch.bfloat16, torch.float32, seed=100 + gi)
            g = mlc.OuterGroup([w.to(DEV) for w in ws0], tg0.to(DEV), u0.to(DEV))
            if quant_bits:
                g.codes = [torch.full((cnt * m, n * quant_bits // 8), 0xAA, dtype=torch.uint8, device=DEV) for _ in range(K)]
                g.scales = [torch.full((cnt * m,), -1.0, dtype=torch.float32, device=DEV) for _ in range(K)]
            if ef:
                g.residuals = [S.normal((cnt, m, n), 1e-3, 100 + gi, 50 + k).to(DEV) for k in range(K)]
            groups.append(g)
        return groups

    together, apart = build(), build()
    mlc.muloco_outer_step(together, hp)              # six groups: one launch of four, then single ones
    for g in apart:
        mlc.muloco_outer_step([g], hp)
    torch.cuda.synchronize()
    for a, b in zip(together, apart):
        assert torch.equal(a.global_param, b.global_param) and torch.equal(a.outer_momentum, b.outer_momentum)
        for k in range(K):
            assert torch.equal(a.worker_params[k].view(torch.int16), b.worker_params[k].view(torch.int16))
            if quant_bits:
                assert torch.equal(a.codes[k], b.codes[k])
                assert torch.equal(a.scales[k].view(torch.int32), b.scales[k].view(torch.int32))
            if ef:
                assert torch.equal(a.residuals[k].view(torch.int32), b.residuals[k].view(torch.int32))
