"""One training step of the L layers that share an expert pool, as a sequence of C-ABI calls.

Nothing here computes: it owns the device buffers (torch is the allocator) and fixes the call
order  route -> permute -> expert_ffn_fwd -> combine  per layer,  pool_aux_loss  once, then
combine_bwd -> expert_ffn_bwd -> combine(unit gates) -> route_bwd  per layer, and the pool
weight gradient either inside every layer call (`wgrad="layer"`) or once at the end over all
layers (`wgrad="pool"`, one long reduction per expert; same result)."""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional

import torch

from . import binding as B


@dataclass
class LayerState:
    topk_idx: torch.Tensor
    topk_gate: torch.Tensor
    logits: torch.Tensor
    x_perm: torch.Tensor
    offsets: torch.Tensor
    row_of_slot: torch.Tensor
    slot_of_row: torch.Tensor
    act_a: torch.Tensor
    act_b: torch.Tensor
    act_h: torch.Tensor
    y_perm: torch.Tensor
    out: torch.Tensor
    # backward
    dy_perm: Optional[torch.Tensor] = None
    d_act: Optional[torch.Tensor] = None
    dx_perm: Optional[torch.Tensor] = None
    dgate: Optional[torch.Tensor] = None
    dx: Optional[torch.Tensor] = None
    d_w_router: Optional[torch.Tensor] = None
    d_sigma: Optional[torch.Tensor] = None


class PoolStep:
    """Sequences the entry points over the L layers that share the pool.

    wgrad     "pool": one weight-gradient pass over all layers at the end of the backward pass;
              "layer": accumulate into the float gradients layer by layer.
    recompute keep one shared pair of A / B buffers instead of one per layer and rebuild a layer's
              A and B (unipool_expert_ffn_recompute) right before its backward pass (App. D (hyperparameter details):
              activation checkpointing with MoE recompute).  Results are bit-identical.
    aux       "pool": the pool-level loss (Eq. 5) over all L layers; "layer": the per-layer loss
              (Eq. 3) for every layer on its own, each with weight one (the ablation row "shared pool
              + layer aux"): unipool_pool_aux_loss is then called once per layer with L = 1, the losses
              are in loss_layers[L] and every layer's backward pass gets its own coefficients.
    router    "norm": the NormRouter of Eq. 7; "softmax": the softmax router of the comparison rows (Sec. 5.4).
    lagged    App. G (pool auxiliary loss derivation), one-step-behind: micro-batch m uses the usage statistic fbar of micro-batch
              m-1, held constant; the first micro-batch uses its own.  The statistic lives in two
              device buffers used in turn and is part of state_dict()."""

    def __init__(self, T, d_model, d_ff, E, k, L, dtype, c, eps, alpha_pool, device="cuda:0",
                 wgrad="pool", recompute=False, lagged=False, aux="pool", router="norm"):
        assert wgrad in ("pool", "layer") and aux in ("pool", "layer") and router in ("norm", "softmax")
        self.router = B.ROUTER_SOFTMAX if router == "softmax" else B.ROUTER_NORM
        assert not (lagged and aux == "layer"), "the lagged statistic belongs to the pool loss"
        self.aux = aux
        self.recompute, self.lagged = bool(recompute), bool(lagged)
        self.micro_batches_done = 0
        self.T, self.d, self.f, self.E, self.k, self.L = T, d_model, d_ff, E, k, L
        self.dtype = dtype
        self.c, self.eps, self.alpha = c, eps, alpha_pool
        self.dev = torch.device(device)
        self.wgrad = wgrad
        self.timing = False          # when set, HIP events bracket every entry point on its stream
        self.events = []             # (entry point, start event, end event)
        self.act = torch.bfloat16 if dtype == B.BF16 else torch.float32
        self.S = T * k
        self.ws = torch.empty(B.workspace_bytes(self.shape(1.0)), dtype=torch.uint8, device=self.dev)
        i32 = dict(dtype=torch.int32, device=self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        act = dict(dtype=self.act, device=self.dev)
        S, f, d = self.S, d_ff, d_model
        self.counts = torch.zeros((L, E), **i32)
        self.psum = torch.zeros((L, E), **f32)
        self.pool_counts = torch.zeros(E, **i32)
        self._fbar2 = [torch.zeros(E, **f32), torch.zeros(E, **f32)]
        self.fbar = self._fbar2[0]           # fbar of the micro-batch that ran last
        self.loss = torch.zeros(1, **f32)
        self.aux_coef = torch.zeros(E, **f32)
        if aux == "layer":
            self.loss_layers = torch.zeros(L, **f32)
            self.aux_coef_layers = torch.zeros((L, E), **f32)
            self.f_layers = torch.zeros((L, E), **f32)
            self._pool_counts_layers = torch.zeros((L, E), **i32)
        self.layers: List[LayerState] = []
        shared_ab = (torch.empty((S, f), **act), torch.empty((S, f), **act)) if self.recompute else None
        for _ in range(L):
            st = LayerState(
                topk_idx=torch.empty((T, k), **i32), topk_gate=torch.empty((T, k), **f32),
                logits=torch.empty((T, E), **f32), x_perm=torch.empty((S, d), **act),
                offsets=torch.empty(E + 1, **i32), row_of_slot=torch.empty((T, k), **i32),
                slot_of_row=torch.empty(S, **i32),
                act_a=shared_ab[0] if self.recompute else torch.empty((S, f), **act),
                act_b=shared_ab[1] if self.recompute else torch.empty((S, f), **act),
                act_h=torch.empty((S, f), **act),
                y_perm=torch.empty((S, d), **act), out=torch.empty((T, d), **act))
            st.dgate = torch.empty((T, k), **f32)
            st.dx = torch.empty((T, d), **act)
            st.d_w_router = torch.empty((E, d), **f32)
            st.d_sigma = torch.empty(1, **f32)
            self.layers.append(st)
        # backward buffers: per layer when the weight gradient is deferred, shared otherwise
        nb = L if wgrad == "pool" else 1
        self._dy = [torch.empty((S, d), **act) for _ in range(nb)]
        self._dact = [torch.empty((S, 2 * f), **act) for _ in range(nb)]
        self._dxp = torch.empty((S, d), **act)
        self.d_w_gate_up = torch.zeros((E, 2 * f, d), **f32)
        self.d_w_down = torch.zeros((E, d, f), **f32)
        if wgrad == "pool":
            def tab(ts):
                return torch.tensor([t.data_ptr() for t in ts], dtype=torch.int64, device=self.dev)
            self._tabs = (tab([s.x_perm for s in self.layers]), tab(self._dact),
                          tab([s.act_h for s in self.layers]), tab(self._dy),
                          tab([s.offsets for s in self.layers]))

    def shape(self, sigma: float, L=None) -> B.Shape:
        return B.Shape(T=self.T, d_model=self.d, d_ff=self.f, E=self.E, k=self.k, L=self.L if L is None else L,
                       dtype=self.dtype, sigma=float(sigma), c=self.c, eps=self.eps,
                       alpha_pool=self.alpha, router=self.router)

    def _call(self, fn, *args):
        if not self.timing:
            return fn(*args)
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()                  # torch's current stream is the one the binding launches on
        fn(*args)
        e1.record()
        self.events.append((fn.__name__, e0, e1))

    # ------------------------------------------------------------------ forward
    def forward_layer(self, l, x, w_router, sigma, w_gate_up, w_down, gather=False):
        """gather: forward-only dispatch without a permuted copy (index maps only; the first GEMM reads the rows
        of x through slot_of_row).  The backward pass needs x_perm, so a training step leaves it off."""
        st, sh, ws = self.layers[l], self.shape(sigma), self.ws
        self._call(B.route, sh, x, w_router, st.topk_idx, st.topk_gate, st.logits, self.counts[l], self.psum[l], ws)
        self._call(B.permute, sh, None if gather else x, st.topk_idx, self.counts[l], None if gather else st.x_perm,
                   st.offsets, st.row_of_slot, st.slot_of_row, ws)
        if gather:
            self._call(B.expert_ffn_fwd_gather, sh, x, st.slot_of_row, st.offsets, w_gate_up, w_down, st.act_a,
                       st.act_b, st.act_h, st.y_perm, ws)
        else:
            self._call(B.expert_ffn_fwd, sh, st.x_perm, st.offsets, w_gate_up, w_down, st.act_a, st.act_b, st.act_h,
                       st.y_perm, ws)
        self._call(B.combine, sh, st.y_perm, st.row_of_slot, st.topk_gate, st.out, ws)
        return st.out

    def aux_loss(self, fbar_in=None):
        """Pool loss of the layers run so far.  In lagged mode the statistic of the previous
        micro-batch is used (none given, none run yet: the current one) and the new one is kept."""
        if self.aux == "layer":
            sh1 = self.shape(1.0, L=1)
            for l in range(self.L):
                self._call(B.pool_aux_loss, sh1, self.counts[l:l + 1], self.psum[l:l + 1], None,
                           self._pool_counts_layers[l], self.f_layers[l], self.loss_layers[l:l + 1],
                           self.aux_coef_layers[l], self.ws)
            self.micro_batches_done += 1
            return self.loss_layers
        out = self.fbar
        if self.lagged:
            if fbar_in is None and self.micro_batches_done > 0:
                fbar_in = self._fbar2[(self.micro_batches_done - 1) % 2]
            out = self._fbar2[self.micro_batches_done % 2]
        self._call(B.pool_aux_loss, self.shape(1.0), self.counts, self.psum, fbar_in, self.pool_counts, out,
                        self.loss, self.aux_coef, self.ws)
        self.fbar = out
        self.micro_batches_done += 1
        return self.loss

    def state_dict(self):
        """What a checkpoint of the micro-batch loop has to hold."""
        return {"micro_batches_done": self.micro_batches_done, "fbar": self.fbar.detach().cpu().clone()}

    def load_state_dict(self, state):
        self.micro_batches_done = int(state["micro_batches_done"])
        if self.micro_batches_done > 0:
            self._fbar2[(self.micro_batches_done - 1) % 2].copy_(state["fbar"].to(self.dev))
            self.fbar = self._fbar2[(self.micro_batches_done - 1) % 2]

    # ------------------------------------------------------------------ backward
    def begin_backward(self):
        if self.wgrad == "layer":
            self.d_w_gate_up.zero_()
            self.d_w_down.zero_()

    def backward_layer(self, l, x, w_router, sigma, w_gate_up, w_down, grad_out):
        st, sh, ws = self.layers[l], self.shape(sigma), self.ws
        slot = l if self.wgrad == "pool" else 0
        dy, dact = self._dy[slot], self._dact[slot]
        self._call(B.combine_bwd, sh, grad_out, st.y_perm, st.row_of_slot, st.topk_gate, dy, st.dgate, ws)
        if self.recompute:
            self._call(B.expert_ffn_recompute, sh, st.x_perm, st.offsets, w_gate_up, st.act_a, st.act_b,
                       st.act_h, ws)
        dwgu = None if self.wgrad == "pool" else self.d_w_gate_up
        dwd = None if self.wgrad == "pool" else self.d_w_down
        self._call(B.expert_ffn_bwd, sh, dy, st.x_perm, st.act_a, st.act_b, st.act_h, st.offsets, w_gate_up, w_down,
                         self._dxp, dact, dwgu, dwd, ws)
        self._call(B.combine, sh, self._dxp, st.row_of_slot, None, st.dx, ws)            # backward of the dispatch
        coef = self.aux_coef if self.aux == "pool" else self.aux_coef_layers[l]
        self._call(B.route_bwd, sh, x, w_router, st.logits, st.topk_idx, st.dgate, coef, st.d_w_router,
                    st.d_sigma, st.dx, True, ws)
        return st.dx

    def end_backward(self):
        if self.wgrad == "pool":
            self._call(B.expert_wgrad, self.shape(1.0), self.L, *self._tabs, self.d_w_gate_up, self.d_w_down,
                           False, self.ws)

    # ------------------------------------------------------------------ whole step
    def step(self, xs, w_routers, sigmas, w_gate_up, w_down, grad_outs, fbar_in=None):
        for l in range(self.L):
            self.forward_layer(l, xs[l], w_routers[l], sigmas[l], w_gate_up, w_down)
        self.aux_loss(fbar_in)
        self.begin_backward()
        for l in reversed(range(self.L)):
            self.backward_layer(l, xs[l], w_routers[l], sigmas[l], w_gate_up, w_down, grad_outs[l])
        self.end_backward()


    # ------------------------------------------------------------------ the step as a HIP graph
    def capture(self, xs, w_routers, sigmas, w_gate_up, w_down, grad_outs):
        """Records one whole step into a HIP graph and returns it (replay() launches it).  The entry points
        allocate nothing, never synchronise and record no memset, so a step is a fixed chain of kernel
        launches on the caller's stream; the graph reads and writes the very buffers given here and the
        step's own state.  Not for the lagged statistic, whose buffers change from one micro-batch to the
        next, nor with event timing on."""
        assert not self.lagged and not self.timing, "a recorded step has fixed buffers and no events"
        # every kernel must have run once outside the recording: their first launch sets function attributes
        self.step(xs, w_routers, sigmas, w_gate_up, w_down, grad_outs)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step(xs, w_routers, sigmas, w_gate_up, w_down, grad_outs)
        return graph


class PoolGroups:
    """Sharing scope G (Sec. 5.4): the layers are cut into G groups over depth and every group has a
    pool, a pool loss and a weight gradient of its own.  One PoolStep per group; a step runs them one
    after the other (group g's weights are w_gate_up[g], w_down[g])."""

    def __init__(self, G, T, d_model, d_ff, E, k, L, dtype, c, eps, alpha_pool, device="cuda:0", **kw):
        assert L % G == 0, "groups hold the same number of layers"
        self.G, self.Lg = G, L // G
        self.groups = [PoolStep(T, d_model, d_ff, E, k, self.Lg, dtype, c, eps, alpha_pool, device=device, **kw)
                       for _ in range(G)]

    def step(self, xs, w_routers, sigmas, w_gate_up, w_down, grad_outs):
        for g, ps in enumerate(self.groups):
            lo, hi = g * self.Lg, (g + 1) * self.Lg
            ps.step(xs[lo:hi], w_routers[lo:hi], sigmas[lo:hi], w_gate_up[g], w_down[g], grad_outs[lo:hi])
