"""A whole step recorded into a HIP graph (the entry points allocate nothing, never synchronise and record
no memset): every replay, with eager steps and synchronisations in between, gives bit for bit what the
eager step gives on the same inputs, also after the inputs have changed in place."""
import pytest

from synth import workloads as W

pytestmark = pytest.mark.gpu

CASES = [
    W.Workload("graph-bf16", L=3, E=24, d=128, f=192, k=2, T=700, dtype="bf16", seed=61, c=2.5, skew="hot"),
    W.Workload("graph-f32", L=2, E=6, d=40, f=48, k=3, T=150, dtype="f32", seed=62, c=2.0),
]


def _outputs(ps):
    outs = [ps.loss, ps.aux_coef, ps.counts, ps.psum, ps.d_w_gate_up, ps.d_w_down]
    for st in ps.layers:
        outs += [st.out, st.dx, st.d_w_router, st.d_sigma, st.topk_idx, st.topk_gate]
    return [o.clone() for o in outs]


@pytest.mark.parametrize("w", CASES, ids=[c.name for c in CASES])
def test_recorded_step_replays_like_the_eager_step(w):
    import torch
    import paper_2605_06665_amd as U
    from paper_2605_06665_amd.pipeline import PoolStep
    dev = torch.device("cuda:0")
    dtype = U.BF16 if w.dtype == "bf16" else U.F32
    xs = [W.gen_x_torch(w, l, dev) for l in range(w.L)]
    wrs = [W.gen_w_router_torch(w, l, dev) for l in range(w.L)]
    gs = [W.gen_grad_out_torch(w, l, dev) for l in range(w.L)]
    wg, wu, wd = W.gen_pool_weights_torch(w, dev)
    wgu = torch.cat([wg, wu], dim=1).contiguous()
    sigmas = [w.sigma + 0.05 * l for l in range(w.L)]
    ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, dtype, w.c, w.eps, w.alpha, device=dev)
    graph = ps.capture(xs, wrs, sigmas, wgu, wd, gs)
    for rep in range(3):
        if rep:                                   # new inputs in the same buffers: the graph reads them in place
            for l in range(w.L):
                xs[l].copy_(torch.roll(xs[l], shifts=rep, dims=0))
                gs[l].mul_(0.5)
        ps.step(xs, wrs, sigmas, wgu, wd, gs)     # eager
        torch.cuda.synchronize()
        want = _outputs(ps)
        for o in (ps.loss, ps.d_w_gate_up, ps.d_w_down, *[st.out for st in ps.layers], *[st.dx for st in ps.layers]):
            o.fill_(float("nan"))                 # what the replay does not write would show
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = _outputs(ps)
        for a, b in zip(got, want):
            assert torch.equal(a, b), "replay %d differs from the eager step" % rep
