"""GPU parity: muloco_adamw_step (C-ABI) against the fp64 oracle over several steps."""
import numpy as np
import pytest
import torch

import paper_2505_23725_amd as mlc
import synth_inputs as S
from oracle import adamw
from helpers import assert_fp32_close, assert_stored_close, to_f64

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

CASES = [
    # elements, param dtype, grad dtype, bias correction
    (4096, torch.float32, torch.float32, False),
    (50257 * 3, torch.bfloat16, torch.bfloat16, True),      # not a multiple of 8: scalar path
    (768 * 1024, torch.bfloat16, torch.float32, True),
    (1000, torch.float32, torch.bfloat16, False),
    (7, torch.float32, torch.float32, True),
]


@pytest.mark.parametrize("n,pd,gd,bc", CASES)
def test_adamw_steps_match_oracle(n, pd, gd, bc):
    th0 = S.normal((n,), S.PARAM_STD, n, 0, dtype=pd)
    th = th0.to(DEV)
    m = torch.zeros(n, dtype=torch.float32, device=DEV)
    v = torch.zeros(n, dtype=torch.float32, device=DEV)
    rth, rm, rv = to_f64(th0), np.zeros(n), np.zeros(n)
    kw = dict(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    for t in range(1, 5):
        g0 = S.normal((n,), S.GRAD_STD, n, 10 + t, dtype=gd)
        start = to_f64(th.cpu())          # both sides start each step from the stored parameters
        mlc.muloco_adamw_step([(th, g0.to(DEV), m, v)], mlc.AdamWHParams(bias_correction=bc, step=t, **kw))
        torch.cuda.synchronize()
        rth, rm, rv = adamw.adamw_step(start, rm, rv, to_f64(g0), step=t, bias_correction=bc, **kw)
        assert_fp32_close(m.cpu(), rm, f"first moment, step {t}")
        assert_fp32_close(v.cpu(), rv, f"second moment, step {t}")
        assert_stored_close(th.cpu(), rth, f"parameters, step {t}")


def test_adamw_several_tensors_in_one_call_and_zero_gradient():
    sizes = [1024, 24, 4104]
    ps = [S.normal((n,), 1.0, 5, i).to(DEV) for i, n in enumerate(sizes)]
    p0 = [p.cpu().clone() for p in ps]
    zs = [torch.zeros(n, device=DEV) for n in sizes]
    ms = [torch.zeros(n, device=DEV) for n in sizes]
    vs = [torch.zeros(n, device=DEV) for n in sizes]
    mlc.muloco_adamw_step(list(zip(ps, zs, ms, vs)), mlc.AdamWHParams(lr=0.1, weight_decay=0.5))
    torch.cuda.synchronize()
    for p, q in zip(ps, p0):          # zero gradient: pure decoupled decay
        assert_fp32_close(p.cpu(), to_f64(q) * (1 - 0.05), "decay only")
    assert all(torch.count_nonzero(x) == 0 for x in ms + vs)
