"""GPU parity at the depth the benchmark runs: workload C5 with all L = 24 layers sharing the pool, in
bench.py's launch configuration (whole steps through the step driver, pooled weight gradient walking
24 layers per expert), and a full-width ragged case (d = 1536, f = 4096, Zipf routing, experts that are
empty in some layers and in all layers).

Integer results, the router and the pool loss are compared in full for every layer.  The expert path is
compared on whole experts: every row an expert received in every layer (so the first and last row of the
expert and the rows on both sides of every row-tile cut are in), and the expert's complete pooled weight
gradient, with the expectations taken from the oracle's expert_ffn_fwd / expert_ffn_bwd on that expert's
rows (from the GPU's own upstream tensors, so that each kernel is judged on its own arithmetic)."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import TOL, check_selection, host, rel_err

pytestmark = pytest.mark.gpu

RAGGED = W.Workload("C5-width-zipf-ragged", L=6, E=192, d=1536, f=4096, k=2, T=3000, dtype="bf16", seed=41,
                    c=3.847, alpha=2e-2, skew="zipf")


def f64(t):
    return host(t).astype(np.float64)


class Step:
    """One whole step on the device, kept for the tests of this module."""

    def __init__(self, w):
        import torch
        import paper_2605_06665_amd as U
        from paper_2605_06665_amd.pipeline import PoolStep
        self.w = w
        dev = torch.device("cuda:0")
        self.dev = dev
        self.xs = [W.gen_x_torch(w, l, dev) for l in range(w.L)]
        self.wrs = [W.gen_w_router_torch(w, l, dev) for l in range(w.L)]
        self.gs = [W.gen_grad_out_torch(w, l, dev) for l in range(w.L)]
        self.wg, self.wu, self.wd = W.gen_pool_weights_torch(w, dev)
        wgu = torch.cat([self.wg, self.wu], dim=1).contiguous()
        self.sig = [1.0 + 0.01 * l for l in range(w.L)]
        self.ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, U.BF16, w.c, w.eps, w.alpha, device=dev, wgrad="pool")
        self.ps.step(self.xs, self.wrs, self.sig, wgu, self.wd, self.gs)
        torch.cuda.synchronize()
        self.offsets = [host(st.offsets).astype(np.int64) for st in self.ps.layers]


@pytest.fixture(scope="module")
def c5_step():
    s = Step(W.WORKLOADS["C5"])          # all 24 layers, as bench.py runs it
    yield s
    del s


@pytest.fixture(scope="module")
def ragged_step():
    s = Step(RAGGED)
    yield s
    del s


def check_router_integers_loss(s, bwd_layers):
    import torch
    w, ps = s.w, s.ps
    tol = TOL[w.dtype]
    T, k, E = w.T, w.k, w.E
    rng = np.random.default_rng(7)
    counts_gpu, psum_gpu, counts_own, n_tie = [], [], [], 0
    for l in range(w.L):
        st = ps.layers[l]
        x, wr = f64(s.xs[l]), f64(s.wrs[l])
        r = O.route(x, wr, k, s.sig[l], w.c, w.eps)
        gi = host(st.topk_idx)
        tie, merged = check_selection(r["z"], r["idx"], gi, k, scores=r["s"], got_gate=host(st.topk_gate), tol=tol)
        n_tie += int(tie.sum())
        assert tie.mean() < 1e-2
        assert rel_err(host(st.logits), r["z"]) <= tol
        gcounts = host(ps.counts[l])
        assert np.array_equal(gcounts, np.bincount(gi.ravel(), minlength=E)) and int(gcounts.sum()) == T * k
        if np.array_equal(gi, r["idx"]):
            assert np.array_equal(gcounts, r["counts"])           # the oracle's own counts
        assert rel_err(host(ps.psum[l]), r["psum"]) <= tol
        counts_gpu.append(gcounts)
        psum_gpu.append(host(ps.psum[l]))
        counts_own.append(r["counts"])
        # permutation: in full, bit exact
        off, ros, sor = O.permutation(gi, E)
        assert np.array_equal(host(st.offsets), off)
        assert np.array_equal(host(st.row_of_slot), ros)
        assert np.array_equal(host(st.slot_of_row), sor)
        # row copies, bitwise: random rows plus the first and last row of every expert
        edge = np.concatenate([off[:-1][np.diff(off) > 0], off[1:][np.diff(off) > 0] - 1])
        rows = np.unique(np.concatenate([rng.choice(w.S, size=256, replace=False), edge]))
        xp = st.x_perm[torch.from_numpy(rows).to(s.dev)]
        assert torch.equal(xp, s.xs[l][torch.from_numpy(sor[rows] // k).to(s.dev)])
        if l in bwd_layers:      # router gradients in full, from the GPU's dgate and coefficients
            dxr, dwr, dsig, _ = O.route_bwd(x, wr, host(st.logits), gi, host(st.dgate), f64(ps.aux_coef),
                                            s.sig[l], w.c, w.eps)
            assert rel_err(host(st.d_w_router), dwr) <= tol, l
            assert abs(float(host(st.d_sigma)[0]) - dsig) <= tol * max(abs(dsig), 1e-3), l
    pc, fbar, loss, coef = O.pool_aux_loss(np.stack(counts_gpu), np.stack(psum_gpu), T, k, w.alpha)
    assert np.array_equal(host(ps.pool_counts), pc) and int(pc.sum()) == w.L * T * k
    assert rel_err(host(ps.fbar), fbar) <= 1e-6 and rel_err(host(ps.aux_coef), coef) <= 1e-6
    assert abs(float(host(ps.loss)[0]) - loss) <= 1e-5 * abs(loss)
    return n_tie


def check_experts(s, experts, fwd_layers):
    """Every row of the given experts in every layer, and their complete pooled weight gradients."""
    w, ps = s.w, s.ps
    tol = TOL[w.dtype]
    f = w.f
    for e in experts:
        wg1, wu1, wd1 = f64(s.wg[e])[None], f64(s.wu[e])[None], f64(s.wd[e])[None]
        dwg, dwu, dwd = np.zeros_like(wg1[0]), np.zeros_like(wu1[0]), np.zeros_like(wd1[0])
        total = 0
        for l in range(w.L):
            st = ps.layers[l]
            r0, r1 = int(s.offsets[l][e]), int(s.offsets[l][e + 1])
            n = r1 - r0
            if n == 0:
                continue
            total += n
            one = np.array([0, n])
            xp, a, b = f64(st.x_perm[r0:r1]), f64(st.act_a[r0:r1]), f64(st.act_b[r0:r1])
            dy = f64(ps._dy[l][r0:r1])
            if l in fwd_layers:
                ra, rb, rh, ry = O.expert_ffn_fwd(xp, one, wg1, wu1, wd1)
                for got, ref, nm in ((a, ra, "a"), (b, rb, "b"), (f64(st.act_h[r0:r1]), rh, "h"),
                                     (f64(st.y_perm[r0:r1]), ry, "y")):
                    assert rel_err(got, ref) <= tol, (e, l, nm)
            dx, g1, g2, g3, da, db = O.expert_ffn_bwd(dy, xp, a, b, one, wg1, wu1, wd1)
            dact = f64(ps._dact[l][r0:r1])
            assert rel_err(dact[:, :f], da) <= tol, (e, l, "dA")
            assert rel_err(dact[:, f:], db) <= tol, (e, l, "dB")
            if l == 0:          # the driver's dx_perm buffer still holds layer 0 (processed last)
                assert rel_err(f64(ps._dxp[r0:r1]), dx) <= tol, (e, "dx_perm")
            dwg += g1[0]
            dwu += g2[0]
            dwd += g3[0]
        got_gu, got_d = f64(ps.d_w_gate_up[e]), f64(ps.d_w_down[e])
        if total == 0:
            assert not got_gu.any() and not got_d.any(), (e, "an expert without rows in any layer has zero gradient")
            continue
        assert rel_err(got_gu, np.concatenate([dwg, dwu], axis=0)) <= tol, (e, "dw_gate_up")
        assert rel_err(got_d, dwd) <= tol, (e, "dw_down")


def test_c5_all_24_layers_router_integers_loss(c5_step):
    assert c5_step.w.L == 24
    check_router_integers_loss(c5_step, bwd_layers=(0, 11, 23))


def test_c5_all_24_layers_whole_experts(c5_step):
    s = c5_step
    tot = host(s.ps.pool_counts)
    order = np.argsort(tot, kind="stable")
    rng = np.random.default_rng(99)
    picks = [int(order[-1]), int(order[0]), int(rng.integers(0, s.w.E))]
    check_experts(s, sorted(set(picks)), fwd_layers=(0, 23))


def test_full_width_ragged_router_integers_loss(ragged_step):
    check_router_integers_loss(ragged_step, bwd_layers=(0, ragged_step.w.L - 1))


def test_full_width_ragged_whole_experts(ragged_step):
    s = ragged_step
    w = s.w
    per_layer = np.stack([np.diff(o) for o in s.offsets])            # [L, E]
    tot = per_layer.sum(axis=0)
    order = np.argsort(tot, kind="stable")
    picks = {int(order[-1])}                                         # hottest: several row tiles per layer
    some_empty = np.where((per_layer == 0).any(axis=0) & (tot > 0))[0]
    assert len(some_empty) > 0, "the ragged case is meant to leave experts empty in some layers"
    picks.add(int(some_empty[0]))
    picks.add(int(some_empty[-1]))
    never = np.where(tot == 0)[0]
    if len(never):
        picks.add(int(never[0]))
    mid = [int(e) for e in order if 16 < per_layer[:, e].max() < 200]
    if mid:
        picks.add(mid[len(mid) // 2])
    check_experts(s, sorted(picks), fwd_layers=tuple(range(w.L)))
