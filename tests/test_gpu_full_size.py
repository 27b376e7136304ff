"""GPU parity at the workloads' full shapes, in the launch configuration bench.py times
(whole shape groups batched per launch, inputs drawn on the GPU), on sampled outputs the
oracle can compute one by one: one matrix per shape group for the Muon inner step, sampled
rows plus one whole matrix per group for the quantised outer step."""
import math

import numpy as np
import pytest
import torch

import paper_2505_23725_amd as mlc
import synth_inputs as S
from oracle import diloco, muon, storage
from helpers import (NS_TOL, assert_fp32_close, assert_ns_close, assert_stored_close, assert_update_elements,
                     rel_fro, to_f64, update_error_bf16)
from paper_2505_23725_amd.harness import MulocoJob

pytestmark = pytest.mark.gpu


def _inner_step_sampled(job: MulocoJob, samples):
    """Run one inner step on the whole job; check the sampled (group, index) matrices."""
    job.draw_gradients(0)
    # non-zero momentum so that the look-ahead matters
    for gi, t in enumerate(job.mom[0]):
        t.copy_(S.normal(tuple(t.shape), 3 * S.GRAD_STD, 0, 700 + gi, device=t.device))
    before = {}
    for (gi, idx) in samples:
        before[(gi, idx)] = (job.workers[0][gi][idx].cpu().clone(), job.grad[0][gi][idx].cpu().clone(),
                             job.mom[0][gi][idx].cpu().clone())
    hp = job.muon_hparams()
    mlc.muloco_inner_step(job.inner_groups(0), hp, job.workspace)
    torch.cuda.synchronize()
    worst = 0.0
    for (gi, idx), (W0, g, m0) in before.items():
        _, m, n = job.shapes[gi]
        w1, m1, o1 = muon.inner_step(to_f64(W0), to_f64(m0), to_f64(g), eta=hp.eta,
                                     weight_decay=hp.weight_decay, beta=hp.beta, nesterov=True,
                                     lr_scale=job.lr_scale(m, n))
        assert_fp32_close(job.mom[0][gi][idx].cpu(), m1, f"group {gi} matrix {idx}: momentum")
        if job.pdtype == torch.bfloat16:     # storage rounding of W removed in quadrature
            err = update_error_bf16(job.workers[0][gi][idx].cpu(), to_f64(W0), w1)
        else:
            err = rel_fro(to_f64(job.workers[0][gi][idx].cpu()) - to_f64(W0), w1 - to_f64(W0))
        worst = max(worst, err)
        assert err <= NS_TOL, f"group {gi} ({m}x{n}) matrix {idx}: update error {err:.3e}"
        assert_update_elements(job.workers[0][gi][idx].cpu(), w1, o1, hp.eta * job.lr_scale(m, n),
                               f"group {gi} ({m}x{n}) matrix {idx}")
    return worst


def test_1p76b_inner_step_sampled_matrices():
    job = MulocoJob(S.WORKLOADS["1.76b"], generate_on="device", seed=0)
    worst = _inner_step_sampled(job, [(0, 5), (0, 95), (1, 3), (2, 23)])
    print(f"1.76B-scale inner step: worst sampled update error {worst:.3e}")


def test_15b_shapes_inner_step_sampled_matrices():
    # the 15B-scale matrix shapes (5120 x 5120, 5120 x 20480, 20480 x 5120) on two layers:
    # the largest K the GEMMs see, with a chunked work space
    wl = S.WORKLOADS["15b"]
    job = MulocoJob(wl, generate_on="device", seed=0, layers=2, workspace_cap_bytes=3 * 2 ** 30)
    worst = _inner_step_sampled(job, [(0, 7), (1, 1), (2, 0)])
    print(f"15B-scale shapes inner step: worst sampled update error {worst:.3e}")


def test_150m_inner_step_all_replicas_batched():
    # 150M-scale, K = 8 replicas resident: one matrix per group on two of the replicas
    wl = S.WORKLOADS["150m"]
    job = MulocoJob(wl, generate_on="device", seed=0)
    job.draw_gradients(0)
    hp = job.muon_hparams()
    picks = [(0, 0, 11), (0, 1, 2), (0, 2, 9), (7, 0, 47), (7, 1, 0), (7, 2, 5)]
    before = {(k, gi, i): (job.workers[k][gi][i].cpu().clone(), job.grad[k][gi][i].cpu().clone())
              for (k, gi, i) in picks}
    job.inner_step()
    torch.cuda.synchronize()
    for (k, gi, i), (W0, g) in before.items():
        _, m, n = job.shapes[gi]
        w1, m1, o1 = muon.inner_step(to_f64(W0), np.zeros((m, n)), to_f64(g), eta=hp.eta,
                                     weight_decay=hp.weight_decay, beta=hp.beta, nesterov=True,
                                     lr_scale=job.lr_scale(m, n))
        err = update_error_bf16(job.workers[k][gi][i].cpu(), to_f64(W0), w1)
        assert err <= NS_TOL, f"replica {k} group {gi} matrix {i}: update error {err:.3e}"
        assert_update_elements(job.workers[k][gi][i].cpu(), w1, o1, hp.eta * job.lr_scale(m, n),
                               f"replica {k} group {gi} matrix {i}")


def test_3p1b_quantised_outer_step_sampled_rows():
    wl = S.WORKLOADS["3.1b"]
    job = MulocoJob(wl, generate_on="device", seed=0, with_quant=True, workspace_cap_bytes=2 ** 30)
    job.displace_workers()
    for gi, u in enumerate(job.u):
        u.copy_(S.normal(tuple(u.shape), 1e-3, 0, 900 + gi, device=u.device))
    K = job.K
    # sampled rows: every 997th row of every group, plus every row of one matrix per group
    picks = {}
    for gi, (c, m, n) in enumerate(job.shapes):
        rows = torch.arange(0, c * m, 997)
        one = torch.arange(m) + (c // 2) * m
        idx = torch.unique(torch.cat([rows, one])).to(job.device)
        picks[gi] = idx
    before = {}
    for gi, idx in picks.items():
        n = job.shapes[gi][2]
        before[gi] = (job.theta_g[gi].reshape(-1, n)[idx].cpu().clone(),
                      job.u[gi].reshape(-1, n)[idx].cpu().clone(),
                      [job.workers[k][gi].reshape(-1, n)[idx].cpu().clone() for k in range(K)])
    hp = job.outer_hparams(quant_bits=4)
    for layer in range(wl.layers):           # the streaming launch configuration of bench.py
        mlc.muloco_outer_step(job.layer_fragment(layer, quant=True), hp)
    torch.cuda.synchronize()
    for gi, idx in picks.items():
        n = job.shapes[gi][2]
        tg0, u0, ws0 = before[gi]
        ref = diloco.outer_step(to_f64(tg0), to_f64(u0), [to_f64(w) for w in ws0], eta_out=hp.eta_out,
                                mu=hp.mu, quant_bits=4)
        for k in range(K):
            got = job.codes[k][gi][idx].cpu().numpy()
            assert np.array_equal(got, diloco.pack_codes4(ref["q"][k])), f"group {gi} worker {k}: codes"
            sc = job.scales[k][gi][idx].cpu().numpy()
            assert np.array_equal(sc.view(np.uint32), ref["scales"][k].view(np.uint32))
        assert_fp32_close(job.u[gi].reshape(-1, n)[idx].cpu(), ref["u"], f"group {gi}: outer momentum")
        assert_fp32_close(job.theta_g[gi].reshape(-1, n)[idx].cpu(), ref["theta"], f"group {gi}: theta_g")
        for k in range(K):
            assert_stored_close(job.workers[k][gi].reshape(-1, n)[idx].cpu(), ref["theta"],
                                f"group {gi} worker {k}: write-back")


def test_150m_fused_outer_step_k8_sampled_rows():
    wl = S.WORKLOADS["150m"]
    job = MulocoJob(wl, generate_on="device", seed=1)
    job.displace_workers()
    picks = {gi: torch.arange(0, c * m, 211).to(job.device) for gi, (c, m, n) in enumerate(job.shapes)}
    before = {gi: (job.theta_g[gi].reshape(-1, job.shapes[gi][2])[idx].cpu().clone(),
                   [job.workers[k][gi].reshape(-1, job.shapes[gi][2])[idx].cpu().clone() for k in range(job.K)])
              for gi, idx in picks.items()}
    job.outer_step()
    torch.cuda.synchronize()
    hp = job.outer_hparams()
    for gi, idx in picks.items():
        n = job.shapes[gi][2]
        tg0, ws0 = before[gi]
        ref = diloco.outer_step(to_f64(tg0), np.zeros(tg0.shape), [to_f64(w) for w in ws0],
                                eta_out=hp.eta_out, mu=hp.mu)
        assert_fp32_close(job.u[gi].reshape(-1, n)[idx].cpu(), ref["u"], "outer momentum")
        assert_fp32_close(job.theta_g[gi].reshape(-1, n)[idx].cpu(), ref["theta"], "theta_g")
        for k in range(job.K):
            assert_stored_close(job.workers[k][gi].reshape(-1, n)[idx].cpu(), ref["theta"], "write-back")


@pytest.mark.parametrize("cnt,m,n", [(3, 2048, 8192), (2, 8192, 2048), (2, 5120, 5120), (1, 2560, 10240)])
def test_newton_schulz_large_shapes(cnt, m, n):
    """The stand-alone entry at the largest shapes of the 1.76B, 3.1B and 15B workloads."""
    x = S.normal((cnt, m, n), S.GRAD_STD, 3, m + n, device="cuda:0", dtype=torch.bfloat16)
    out = torch.empty_like(x)
    ws = torch.empty(mlc.newton_schulz_workspace_bytes(cnt, m, n), dtype=torch.uint8, device="cuda:0")
    mlc.newton_schulz(x, out, ws)
    torch.cuda.synchronize()
    i = cnt - 1
    ref = muon.newton_schulz(to_f64(x[i].cpu()), 5)
    st = assert_ns_close(to_f64(out[i].cpu()), ref, f"NS {m}x{n}")
    print(f"NS {m}x{n}: relative Frobenius error {st['fro']:.3e}, worst 256-block {st['tile']:.3e}, "
          f"largest element error {st['max'] / st['rms']:.1f}x rms")
