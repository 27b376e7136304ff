"""Device-side bookkeeping for running the MuLoCo hot path on a synthetic workload.

Owns the torch tensors (parameters of K worker replicas, Muon momentum, gradients, the
global copy and the outer momentum, quantiser outputs, the work space) and builds the
group descriptors the C-ABI calls take.  It performs no optimizer arithmetic: every
update happens inside libmuloco.so.
"""
from __future__ import annotations

import math
from typing import List, Optional

import torch

import synth_inputs as S
from . import binding as B


class StreamingSchedule:
    """Partitioned communication (paper Sec. 2 "Partitioned Communication in Streaming DiLoCo";
    Sec. 6 "Streaming MuLoCo"): the layers are split into J subsets, J divides the
    communication interval H, and subset j (1 <= j <= J) takes its outer step at the inner
    steps t with t = j * H / J modulo H, so every subset is synchronised once per H steps and
    1 / J of the model at a time.  Subsets are contiguous runs of layers, as equal as L allows."""

    def __init__(self, layers: int, H: int, J: int):
        if J < 1 or H < 1 or H % J != 0:
            raise ValueError("the number of subsets J must divide the communication interval H")
        if J > layers:
            raise ValueError("more subsets than layers")
        self.layers, self.H, self.J = layers, H, J
        bounds = [round(j * layers / J) for j in range(J + 1)]
        self.subsets = [range(bounds[j], bounds[j + 1]) for j in range(J)]

    def due(self, t: int) -> Optional[int]:
        """0-based index of the subset synchronised after inner step t (t counts from 1), or None."""
        every = self.H // self.J
        if t < 1 or t % every != 0:
            return None
        return (t // every - 1) % self.J


class MulocoJob:
    def __init__(self, workload: S.Workload, device="cuda:0", seed: int = 0,
                 layers: Optional[int] = None, K: Optional[int] = None,
                 with_quant: bool = False, quant_bits: int = 4, with_ef: bool = False,
                 workspace_cap_bytes: Optional[int] = None,
                 grad_dtype: Optional[torch.dtype] = None, generate_on: str = "cpu",
                 outer_only: bool = False):
        """generate_on: "cpu" draws every tensor with the CPU generator and copies it over
        (reproducible on the host for parity tests); "device" draws on the GPU (full-size
        workloads).  outer_only: hold only what the outer step touches (no Muon momentum, no
        gradients, no Newton-Schulz work space)."""
        self.wl = workload
        self.device = torch.device(device)
        self.seed = seed
        self.K = workload.K if K is None else K
        L = workload.layers if layers is None else layers
        d, f = workload.d_model, workload.d_ffn
        self.shapes = [(4 * L, d, d), (L, d, f), (L, f, d)]
        self.pdtype = S.torch_dtype(workload.param_dtype)
        self.gdtype = grad_dtype or self.pdtype
        self.gen_dev = "cpu" if generate_on == "cpu" else self.device
        self.theta_g: List[torch.Tensor] = []
        self.u: List[torch.Tensor] = []
        # The K replicas of a shape group are stacked in one [K, count, m, n] tensor, so the
        # inner step can hand all K * count matrices of a shape to the library as one group
        # (one launch per kernel kind); workers[k][gi] etc. are views of replica k.
        self.W: List[torch.Tensor] = []
        self.M: List[torch.Tensor] = []
        self.G: List[torch.Tensor] = []
        self.workers: List[List[torch.Tensor]] = [[] for _ in range(self.K)]
        self.mom: List[List[torch.Tensor]] = [[] for _ in range(self.K)]
        self.grad: List[List[torch.Tensor]] = [[] for _ in range(self.K)]
        for gi, shp in enumerate(self.shapes):
            self.theta_g.append(torch.empty(shp, dtype=torch.float32, device=self.device))
            self.u.append(torch.zeros(shp, dtype=torch.float32, device=self.device))
            self.W.append(torch.empty((self.K,) + tuple(shp), dtype=self.pdtype, device=self.device))
            if not outer_only:
                self.M.append(torch.zeros((self.K,) + tuple(shp), dtype=torch.float32, device=self.device))
                self.G.append(torch.zeros((self.K,) + tuple(shp), dtype=self.gdtype, device=self.device))
            # theta^(0) in the worker dtype, the same for the global copy and every replica
            self._fill([self.theta_g[gi]] + [self.W[gi][k] for k in range(self.K)], shp,
                       S.PARAM_STD, 100 + gi, self.pdtype)
            for k in range(self.K):
                self.workers[k].append(self.W[gi][k])
                if not outer_only:
                    self.mom[k].append(self.M[gi][k])
                    self.grad[k].append(self.G[gi][k])
        self.codes = self.scales = self.residuals = None
        self.quant_bits = quant_bits
        if with_quant:
            self.codes = [[torch.empty((c * m, n * quant_bits // 8), dtype=torch.uint8, device=self.device)
                           for (c, m, n) in self.shapes] for _ in range(self.K)]
            self.scales = [[torch.empty((c * m,), dtype=torch.float32, device=self.device)
                            for (c, m, n) in self.shapes] for _ in range(self.K)]
        if with_ef:      # error-feedback residuals E_k, zero at the start (Algorithm 2)
            self.residuals = [[torch.zeros(shp, dtype=torch.float32, device=self.device)
                               for shp in self.shapes] for _ in range(self.K)]
        self.workspace = None
        if outer_only:
            return
        # room for all shape groups at once: their products of equal depth then share launches
        need = B.muloco_inner_workspace_bytes(self.inner_groups_all())
        floor = max(B.newton_schulz_workspace_min_bytes(s[1], s[2]) for s in self.shapes)
        if workspace_cap_bytes is not None:
            need = max(floor, min(need, workspace_cap_bytes))
        self.workspace = torch.empty(need, dtype=torch.uint8, device=self.device)

    # -- synthetic draws --------------------------------------------------------------
    def _draw(self, shape, std, stream, dtype):
        return S.normal(shape, std, self.seed, stream, device=self.gen_dev, dtype=dtype).to(self.device)

    # Largest number of elements drawn at once on the device: the fp32 temporary of a whole
    # 15B-scale group would not fit beside the resident state.
    DEVICE_DRAW_ELEMS = 1 << 28

    def _fill(self, dsts, shape, std, stream, dtype) -> None:
        """dst.copy_(std * N(0,1) rounded to `dtype`) for every dst.  Drawn on the CPU the
        tensor is one draw of `stream` (what a parity test reproduces on the host); drawn on
        the device it is made of slices along the first dimension, one sub-stream each."""
        count = shape[0]
        per = 1
        for v in shape[1:]:
            per *= v
        step = count if self.gen_dev == "cpu" else max(1, self.DEVICE_DRAW_ELEMS // per)
        if step >= count:
            x = self._draw(shape, std, stream, dtype)
            for d in dsts:
                d.copy_(x)
            return
        for i, c0 in enumerate(range(0, count, step)):
            c1 = min(count, c0 + step)
            x = self._draw((c1 - c0,) + tuple(shape[1:]), std, stream * 65_536 + i + 1_000_000, dtype)
            for d in dsts:
                d[c0:c1].copy_(x)
            del x

    def grad_stream(self, k: int, step: int, gi: int) -> int:
        return 10_000 + (step * 64 + k) * 8 + gi

    def draw_gradients(self, step: int) -> None:
        """Fresh i.i.d. gradients for every replica: g ~ 1e-3 N(0,1), keyed by (k, step, group)."""
        for k in range(self.K):
            for gi, shp in enumerate(self.shapes):
                self._fill([self.grad[k][gi]], shp, S.GRAD_STD, self.grad_stream(k, step, gi), self.gdtype)

    def displace_workers(self, std: float = S.DELTA_STD) -> None:
        """theta_k = theta_g - Delta_k with Delta_k ~ std N(0,1): stands in for H inner steps
        when only the outer step is exercised."""
        for k in range(self.K):
            for gi, shp in enumerate(self.shapes):
                # the replica first receives Delta_k, then theta_g - Delta_k in place
                w = self.workers[k][gi]
                self._fill([w], shp, std, 5_000 + k * 8 + gi, torch.float32)
                step = max(1, self.DEVICE_DRAW_ELEMS // (shp[1] * shp[2]))
                for c0 in range(0, shp[0], step):
                    c1 = min(shp[0], c0 + step)
                    w[c0:c1].copy_(self.theta_g[gi][c0:c1] - w[c0:c1].to(torch.float32))

    # -- descriptors --------------------------------------------------------------------
    @staticmethod
    def lr_scale(m: int, n: int) -> float:
        """Paper Sec. 5 "MuLoCo": rescale the learning rate by sqrt(n/m) for an m x n matrix."""
        return math.sqrt(n / m)

    def inner_groups(self, k: int) -> List[B.InnerGroup]:
        """Groups of replica k only."""
        return [B.InnerGroup(self.workers[k][gi], self.grad[k][gi], self.mom[k][gi],
                             self.lr_scale(m, n))
                for gi, (c, m, n) in enumerate(self.shapes)]

    def inner_groups_all(self) -> List[B.InnerGroup]:
        """One group per shape holding the matrices of all K replicas: K * count matrices."""
        out = []
        for gi, (c, m, n) in enumerate(self.shapes):
            out.append(B.InnerGroup(self.W[gi].view(self.K * c, m, n), self.G[gi].view(self.K * c, m, n),
                                    self.M[gi].view(self.K * c, m, n), self.lr_scale(m, n)))
        return out

    def outer_groups(self, quant: bool = False, group_ids=None, ef: bool = False) -> List[B.OuterGroup]:
        ids = range(len(self.shapes)) if group_ids is None else group_ids
        out = []
        for gi in ids:
            ws = [self.workers[k][gi] for k in range(self.K)]
            g = B.OuterGroup(ws, self.theta_g[gi], self.u[gi])
            if quant:
                g.codes = [self.codes[k][gi] for k in range(self.K)]
                g.scales = [self.scales[k][gi] for k in range(self.K)]
            if ef:
                g.residuals = [self.residuals[k][gi] for k in range(self.K)]
            out.append(g)
        return out

    def layer_fragment(self, layer: int, quant: bool = False, ef: bool = False) -> List[B.OuterGroup]:
        """Outer-step groups covering one transformer layer (4 d x d, one d x f, one f x d)."""
        return self.layers_fragment(range(layer, layer + 1), quant, ef)

    def layers_fragment(self, layers: range, quant: bool = False, ef: bool = False) -> List[B.OuterGroup]:
        """Outer-step groups covering a contiguous run of layers: the unit a streaming schedule
        synchronises at a time."""
        out = []
        l0, l1 = layers.start, layers.stop
        for gi, (c, m, n) in enumerate(self.shapes):
            per_layer = 4 if gi == 0 else 1
            sl = slice(l0 * per_layer, l1 * per_layer)
            ws = [self.workers[k][gi][sl] for k in range(self.K)]
            g = B.OuterGroup(ws, self.theta_g[gi][sl], self.u[gi][sl])
            if quant:
                rows = slice(l0 * per_layer * m, l1 * per_layer * m)
                g.codes = [self.codes[k][gi][rows] for k in range(self.K)]
                g.scales = [self.scales[k][gi][rows] for k in range(self.K)]
            if ef:
                g.residuals = [self.residuals[k][gi][sl] for k in range(self.K)]
            out.append(g)
        return out

    def muon_hparams(self) -> B.MuonHParams:
        return B.MuonHParams(eta=self.wl.eta_in, weight_decay=self.wl.weight_decay, beta=self.wl.beta,
                             nesterov=True)

    def outer_hparams(self, quant_bits: int = 0, write_back: bool = True, error_feedback: bool = False,
                      ef_beta: float = 1.0) -> B.OuterHParams:
        return B.OuterHParams(K=self.K, eta_out=self.wl.eta_out, mu=self.wl.mu, nesterov=True,
                              quant_bits=quant_bits, write_back=write_back,
                              error_feedback=error_feedback, ef_beta=ef_beta)

    # -- the hot path -----------------------------------------------------------------------
    def inner_step(self) -> None:
        """One Muon step of every replica: same-shape matrices of all replicas share launches."""
        B.muloco_inner_step(self.inner_groups_all(), self.muon_hparams(), self.workspace)

    def outer_step(self, quant_bits: int = 0) -> None:
        B.muloco_outer_step(self.outer_groups(quant=quant_bits != 0), self.outer_hparams(quant_bits))

    def run_streaming(self, schedule: StreamingSchedule, steps: int, quant_bits: int = 0, first_step: int = 1,
                      draw: bool = True) -> List[tuple]:
        """`steps` inner steps of every replica with the outer step of the subset that is due
        after each of them (paper Sec. 2 "Partitioned Communication").  Returns the
        (inner step, subset) pairs that were synchronised."""
        hp = self.outer_hparams(quant_bits=quant_bits)
        done = []
        for t in range(first_step, first_step + steps):
            if draw:
                self.draw_gradients(t - 1)
            self.inner_step()
            j = schedule.due(t)
            if j is not None:
                B.muloco_outer_step(self.layers_fragment(schedule.subsets[j], quant=quant_bits != 0), hp)
                done.append((t, j))
        return done

    @staticmethod
    def capture(fn):
        """Record the kernel launches of fn() into a HIP graph and return it (replay()
        re-issues them with one call).  The library's entry points only enqueue kernels on
        the current stream, neither allocating nor synchronising, so they can be captured;
        fn runs once eagerly first (its effects are real) so that one-time set-up such as
        raising a kernel's LDS limit happens outside the capture.  The timing recorder must
        be off: it records events."""
        B.muloco_timing_enable(False)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        return graph

    def ns_flops(self, iters: int = 5) -> float:
        """Nominal Newton-Schulz FLOP (4 s^2 l + 2 s^3 per iteration) of one replica's inner step."""
        tot = 0.0
        for (c, m, n) in self.shapes:
            mp, np_ = -(-m // 128) * 128, -(-n // 128) * 128
            s, l = min(mp, np_), max(mp, np_)
            tot += c * iters * (4.0 * s * s * l + 2.0 * s ** 3)
        return tot
