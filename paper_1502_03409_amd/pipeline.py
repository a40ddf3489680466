"""Host schedule of the layer pipeline of Sec. 3.1 (training paragraph and the figure on semi-parallel training):
every layer L but the last runs as two instances, one that keeps training (`sae_step`, Eq. 1) and a forward-only
one whose parameters are a copy of the training instance's, refreshed every `sync_period` steps; the forward-only
instance turns the mini-batch into the input of layer L+1 (`lc_forward`, then L2 pooling and contrast
normalisation), so layer L+1 trains while layer L is still training.

This module only orders calls of the C ABI on HIP streams: each stage owns one stream of default priority, its
kernels run there in program order, and two kinds of events tie the stages together:

  ready[s][t]   stage s's forward-only instance has written the features of step t (stage s+1 waits for it);
  done[s][t]    stage s has finished reading its input of step t (stage s-1 waits for done[s][t-2] before it
                overwrites that buffer: the features are double-buffered by the parity of t).

With `streams=False` the very same calls are issued on the caller's current stream, stage after stage, which is
the reference the streamed schedule must reproduce bit for bit (every kernel is deterministic).  The refresh of
the forward-only copy is a device-to-device copy on the stage's own stream, between that stage's training steps,
so it never overlaps an update of the weights it reads.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import torch

from . import binding as lc


@dataclass
class PipelineStage:
    """One layer: its training instance (w, b, alpha), and, unless it is the last, its forward-only instance."""

    g: lc.LcGeom
    w: torch.Tensor
    b: torch.Tensor
    alpha: torch.Tensor
    lam: float
    last: bool
    cost: torch.Tensor = None
    ws: torch.Tensor = None
    wf: Optional[torch.Tensor] = None          # forward-only copy of w
    alphaf: Optional[torch.Tensor] = None      # and of alpha
    hf: Optional[torch.Tensor] = None          # forward-only features
    fws: Optional[torch.Tensor] = None         # lc_forward's optional workspace
    p: Optional[torch.Tensor] = None           # pooled
    n: List[torch.Tensor] = field(default_factory=list)   # normalised, one buffer per parity of the step
    mu: Optional[torch.Tensor] = None
    rstd: Optional[torch.Tensor] = None


class SaePipeline:
    """Stages chained as LC layer -> 3x3 L2 pooling -> 5x5 contrast normalisation (the benchmark's chain)."""

    def __init__(self, geoms: Sequence[lc.LcGeom], weights: Sequence[torch.Tensor], biases: Sequence[torch.Tensor],
                 alphas: Sequence[float], lambdas: Sequence[float], *, sync_period: int, eps_sparse: float, lr: float,
                 flags: int, pool=(3, 1, 1e-6), lcn=(5, 1.0, 1e-4), streams: bool = True):
        if sync_period < 1:
            raise ValueError("sync_period must be at least 1")
        self.P, self.eps_sparse, self.lr, self.flags = sync_period, eps_sparse, lr, flags
        self.pool, self.lcn = pool, lcn
        self.stages: List[PipelineStage] = []
        dev = weights[0].device
        for s, g in enumerate(geoms):
            LH, LW, K = lc.geom_derive(g)
            last = s == len(geoms) - 1
            st = PipelineStage(g=g, w=weights[s], b=biases[s], lam=lambdas[s], last=last,
                               alpha=torch.tensor([alphas[s]], device=dev, dtype=torch.float32))
            st.cost = torch.zeros(1, device=dev)
            st.ws = torch.empty(lc.workspace_bytes(g, lc.LC_OP_SAE_STEP), dtype=torch.uint8, device=dev)
            if not last:
                ks, stride, _ = pool
                Hp, Wp = (LH - ks) // stride + 1, (LW - ks) // stride + 1
                st.wf, st.alphaf = torch.empty_like(st.w), torch.empty_like(st.alpha)
                st.hf = torch.empty((g.B, LH, LW, g.F), device=dev)
                nfw = lc.workspace_bytes(g, lc.LC_OP_FORWARD)
                st.fws = torch.empty(nfw, dtype=torch.uint8, device=dev) if nfw else None
                st.p = torch.empty((g.B, Hp, Wp, g.F), device=dev)
                st.n = [torch.empty_like(st.p), torch.empty_like(st.p)]
                st.mu = torch.empty((g.B, Hp, Wp), device=dev)
                st.rstd = torch.empty_like(st.mu)
            self.stages.append(st)
        self.streams = [torch.cuda.Stream(device=dev) for _ in geoms] if streams else None
        self.t = 0
        self._ready = [dict() for _ in geoms]
        self._done = [dict() for _ in geoms]

    # ------------------------------------------------------------------------------------------------ schedule
    def _stage_work(self, s: int, t: int, x_in: torch.Tensor, sm: Optional[torch.cuda.Stream]) -> None:
        """Everything stage s does in step t, in order, on the current stream (sm: that stream when the stages run
        on streams of their own, so that the events other stages wait for can be recorded on it)."""
        st = self.stages[s]
        if not st.last:
            if t % self.P == 0:                       # periodic synchronisation of the forward-only instance
                st.wf.copy_(st.w, non_blocking=True)
                st.alphaf.copy_(st.alpha, non_blocking=True)
            lc.lc_forward_dev_scale(st.g, x_in, st.wf, None, st.alphaf, st.hf, st.fws)
            lc.l2pool_lcn_fwd(st.hf, st.p, st.n[t % 2], st.mu, st.rstd, *self.pool, *self.lcn)
            if sm is not None:
                ev = torch.cuda.Event()
                ev.record(sm)
                self._ready[s][t] = ev
        lc.sae_step(st.g, x_in, st.w, st.b, st.alpha, st.lam, self.eps_sparse, self.lr, self.flags, None, st.cost, st.ws)
        if sm is not None and s > 0:
            ev = torch.cuda.Event()
            ev.record(sm)
            self._done[s][t] = ev

    def step(self, x: torch.Tensor) -> None:
        """One mini-batch through every stage (enqueue only; nothing here synchronises with the host)."""
        t = self.t
        self.t += 1
        if self.streams is None:
            x_in = x
            for s, st in enumerate(self.stages):
                self._stage_work(s, t, x_in, None)
                x_in = None if st.last else st.n[t % 2]
            return
        start = torch.cuda.Event()
        start.record(torch.cuda.current_stream())     # x is ready once the caller's earlier work is
        for s, (st, sm) in enumerate(zip(self.stages, self.streams)):
            if s == 0:
                x_in = x
                sm.wait_event(start)
            else:
                x_in = self.stages[s - 1].n[t % 2]
                sm.wait_event(self._ready[s - 1].pop(t))
            if not st.last and (t - 2) in self._done[s + 1]:
                sm.wait_event(self._done[s + 1].pop(t - 2))   # the buffer this step overwrites has been read
            with torch.cuda.stream(sm):
                self._stage_work(s, t, x_in, sm)

    def join(self) -> None:
        """Make the caller's current stream wait for everything enqueued so far."""
        if self.streams is None:
            return
        caller = torch.cuda.current_stream()
        for sm in self.streams:
            ev = torch.cuda.Event()
            ev.record(sm)
            caller.wait_event(ev)
