"""GPU parity on the smallest workload, whole: a 2-layer d=128 / FFN 512 fp32 parameter set,
K = 1, H = 8 Muon steps (momentum 0.95, Nesterov, 5 Newton-Schulz iterations) with a fresh
seeded gradient per step, then one outer Nesterov step (lr 0.7, momentum 0.9).  The oracle
runs the same trajectory in fp64 from the same seeded draws."""
import numpy as np
import pytest
import torch

import synth_inputs as S
from oracle import diloco, muon
from helpers import NS_TOL, assert_fp32_close, rel_fro, to_f64

pytestmark = pytest.mark.gpu


def test_tiny_workload_h8_then_outer_step():
    from paper_2505_23725_amd.harness import MulocoJob
    wl = S.WORKLOADS["tiny"]
    job = MulocoJob(wl, generate_on="cpu", seed=0)
    theta0 = [t.cpu().clone() for t in job.theta_g]
    for h in range(wl.H):
        job.draw_gradients(h)
        job.inner_step()
    torch.cuda.synchronize()
    W_gpu = [w.cpu() for w in job.workers[0]]
    m_gpu = [m.cpu() for m in job.mom[0]]
    job.outer_step()
    torch.cuda.synchronize()

    worst = 0.0
    for gi, (cnt, m, n) in enumerate(job.shapes):
        th0 = to_f64(S.normal((cnt, m, n), S.PARAM_STD, 0, 100 + gi))
        assert np.array_equal(th0, to_f64(theta0[gi]))
        W = th0.copy()
        mom = np.zeros_like(W)
        for h in range(wl.H):
            g = to_f64(S.normal((cnt, m, n), S.GRAD_STD, 0, job.grad_stream(0, h, gi)))
            for i in range(cnt):
                W[i], mom[i], _ = muon.inner_step(W[i], mom[i], g[i], eta=wl.eta_in,
                                                  weight_decay=wl.weight_decay, beta=wl.beta,
                                                  nesterov=True, lr_scale=job.lr_scale(m, n))
        assert_fp32_close(m_gpu[gi], mom, f"group {gi}: momentum after H steps")
        for i in range(cnt):
            err = rel_fro(to_f64(W_gpu[gi][i]) - th0[i], W[i] - th0[i])
            worst = max(worst, err)
            assert err <= NS_TOL, f"group {gi} matrix {i}: displacement error {err:.3e}"
        # outer step: the oracle starts from the parameters the GPU reached after its H inner
        # steps, so this leg is an elementwise fp32 path and is held to its own tolerance
        out = diloco.outer_step(th0.reshape(-1, n), np.zeros((cnt * m, n)), [to_f64(W_gpu[gi]).reshape(-1, n)],
                                eta_out=wl.eta_out, mu=wl.mu)
        assert_fp32_close(job.u[gi].cpu().reshape(-1, n), out["u"], f"group {gi}: outer momentum")
        assert_fp32_close(job.theta_g[gi].cpu().reshape(-1, n), out["theta"], f"group {gi}: theta_g")
        th_gpu = to_f64(job.theta_g[gi].cpu()).reshape(-1, n)
        assert rel_fro(th_gpu - th0.reshape(-1, n), out["theta"] - th0.reshape(-1, n)) <= 1e-5
        assert torch.equal(job.workers[0][gi], job.theta_g[gi]), "write-back must copy theta_g"
    print(f"tiny workload: worst displacement error after H={wl.H} steps {worst:.3e}")


# bf16 weights and matrices large enough for the batched GEMM kernels (shared launches, the
# update written by the last product), small enough to run in a moment
MID = S.Workload("mid", 40, 256, 1024, K=1, H=4, param_dtype="bf16")


@pytest.mark.parametrize("wl", [S.WORKLOADS["tiny"], MID], ids=["tiny", "mid-bf16"])
def test_graph_replay_equals_eager_steps(wl):
    """The whole step (Muon inner step, outer step, 4-bit quantised outer step per layer) is
    captured into a HIP graph once; replays, with eager work and synchronisations between
    them, must give the bits that the same number of eager steps gives."""
    import paper_2505_23725_amd as mlc
    from paper_2505_23725_amd.harness import MulocoJob

    def make():
        job = MulocoJob(wl, generate_on="cpu", seed=3, K=2, with_quant=True)
        job.draw_gradients(0)
        hp = job.outer_hparams(quant_bits=4)

        def step():
            job.inner_step()
            job.outer_step(0)
            for layer in range(wl.layers):
                mlc.muloco_outer_step(job.layer_fragment(layer, quant=True), hp)
        return job, step

    eager, eager_step = make()
    replayed, replayed_step = make()
    graph = MulocoJob.capture(replayed_step)      # runs the step once eagerly, then records it
    eager_step()
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 16, device="cuda:0")
    for rep in range(3):
        eager_step()
        graph.replay()
        scratch.add_(1.0)                          # unrelated eager work between replays
        torch.cuda.synchronize()
        for gi in range(len(eager.shapes)):
            assert torch.equal(eager.theta_g[gi], replayed.theta_g[gi]), f"replay {rep}: theta_g of group {gi}"
            assert torch.equal(eager.u[gi], replayed.u[gi]), f"replay {rep}: outer momentum of group {gi}"
            assert torch.equal(eager.W[gi], replayed.W[gi]) and torch.equal(eager.M[gi], replayed.M[gi])
            for k in range(eager.K):
                assert torch.equal(eager.codes[k][gi], replayed.codes[k][gi])
                assert torch.equal(eager.scales[k][gi], replayed.scales[k][gi])
    assert float(scratch[0]) == 3.0


def test_streaming_schedule_two_subsets_two_replicas():
    """Partitioned communication (Sec. 2 "Partitioned Communication in Streaming DiLoCo") on the
    smallest workload: K = 2 replicas, H = 8, the two layers as J = 2 subsets, so layer 0 takes its
    outer step after inner step 4 and layer 1 after inner step 8.  The oracle runs the same
    trajectory in fp64 with its own schedule."""
    from paper_2505_23725_amd.harness import MulocoJob, StreamingSchedule
    wl = S.WORKLOADS["tiny"]
    K, J = 2, 2
    job = MulocoJob(wl, generate_on="cpu", seed=0, K=K)
    sch = StreamingSchedule(wl.layers, wl.H, J)
    done = job.run_streaming(sch, wl.H)
    torch.cuda.synchronize()
    assert done == [(t, diloco.streaming_due(t, wl.H, J) - 1) for t in range(1, wl.H + 1)
                    if diloco.streaming_due(t, wl.H, J)] == [(4, 0), (8, 1)]

    worst = 0.0
    for gi, (cnt, m, n) in enumerate(job.shapes):
        per_layer = cnt // wl.layers
        th0 = to_f64(S.normal((cnt, m, n), S.PARAM_STD, 0, 100 + gi))
        theta, u = th0.copy(), np.zeros_like(th0)
        W = [th0.copy() for _ in range(K)]
        mom = [np.zeros_like(th0) for _ in range(K)]
        for t in range(1, wl.H + 1):
            for k in range(K):
                g = to_f64(S.normal((cnt, m, n), S.GRAD_STD, 0, job.grad_stream(k, t - 1, gi)))
                for i in range(cnt):
                    W[k][i], mom[k][i], _ = muon.inner_step(W[k][i], mom[k][i], g[i], eta=wl.eta_in,
                                                            weight_decay=wl.weight_decay, beta=wl.beta,
                                                            nesterov=True, lr_scale=job.lr_scale(m, n))
            j = diloco.streaming_due(t, wl.H, J)
            if j:      # the layers of subset j: contiguous matrices of this group
                sl = slice((j - 1) * per_layer, j * per_layer)
                out = diloco.outer_step(theta[sl].reshape(-1, n), u[sl].reshape(-1, n),
                                        [W[k][sl].reshape(-1, n) for k in range(K)], eta_out=wl.eta_out, mu=wl.mu)
                theta[sl] = out["theta"].reshape(theta[sl].shape)
                u[sl] = out["u"].reshape(u[sl].shape)
                for k in range(K):
                    W[k][sl] = theta[sl]
        for i in range(cnt):
            err = rel_fro(to_f64(job.theta_g[gi][i].cpu()) - th0[i], theta[i] - th0[i])
            worst = max(worst, err)
            assert err <= NS_TOL, f"group {gi} matrix {i}: global displacement error {err:.3e}"
            assert rel_fro(to_f64(job.u[gi][i].cpu()), u[i]) <= NS_TOL
            for k in range(K):
                assert rel_fro(to_f64(job.workers[k][gi][i].cpu()) - th0[i], W[k][i] - th0[i]) <= NS_TOL
        # the subset synchronised last holds theta_g in every replica, bit for bit
        last = slice((J - 1) * per_layer, J * per_layer)
        for k in range(K):
            assert torch.equal(job.workers[k][gi][last], job.theta_g[gi][last])
    print(f"streaming tiny workload: worst global displacement error {worst:.3e}")
