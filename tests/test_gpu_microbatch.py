"""GPU parity of the stateful micro-batch loop: the one-step-behind usage statistic (App. G (pool auxiliary loss derivation)) against
the oracle's loop, its checkpoint, and the recompute mode (App. D (hyperparameter details)), whose results must be bitwise
those of the mode that keeps the activations; and of the sharing-scope variants of Sec. 5.4 (per-layer
loss on the shared pool, pool groups over depth)."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import TOL, check_selection, dev, host, rel_err
from tests.test_gpu_parity import CASES, empty, lib, oracle_case, pack_gate_up, shape_of, workspace, _ffn_inputs

pytestmark = pytest.mark.gpu

RECOMPUTE_CASES = ["C1", "f32-ragged", "bf16-tiles", "bf16-skew", "bf16-empty", "bf16-k8"]
LOOP_CASES = ["C1", "bf16-tiles", "bf16-skew"]


def _act(w):
    U = lib()
    return U.BF16 if w.dtype == "bf16" else U.F32


@pytest.mark.parametrize("name", RECOMPUTE_CASES)
def test_recompute_entry_point(name):
    import torch
    c = oracle_case(name)
    w, U = c["w"], lib()
    sh = shape_of(w)
    r, off, ros, sor, x_perm = _ffn_inputs(c)
    a, b, h = O.expert_ffn_recompute(x_perm, off, c["wg"], c["wu"])
    fa, fb, fh, ra, rb, rh = (empty((w.S, w.f), w.dtype) for _ in range(6))
    fy = empty((w.S, w.d), w.dtype)
    for t in (ra, rb, rh):
        t.fill_(float("nan"))
    gx, goff = dev(x_perm, w.dtype), dev(off.astype(np.int32))
    gwgu, gwd = dev(pack_gate_up(c["wg"], c["wu"]), w.dtype), dev(c["wd"], w.dtype)
    ws = workspace(sh)
    U.expert_ffn_fwd(sh, gx, goff, gwgu, gwd, fa, fb, fh, fy, ws)
    U.expert_ffn_recompute(sh, gx, goff, gwgu, ra, rb, rh, ws)
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    for got, fwd, ref_, nm in ((ra, fa, a, "a"), (rb, fb, b, "b"), (rh, fh, h, "h")):
        assert np.isfinite(host(got)).all(), nm + " has unwritten elements"
        assert torch.equal(got, fwd), nm + ": recomputed values differ from the forward pass's"
        assert rel_err(host(got), ref_) <= tol, nm


@pytest.mark.parametrize("name", RECOMPUTE_CASES)
@pytest.mark.parametrize("wgrad", ["pool", "layer"])
def test_step_with_recompute_is_bitwise_the_same(name, wgrad):
    import torch
    from paper_2605_06665_amd.pipeline import PoolStep
    c = oracle_case(name)
    w = c["w"]
    xs = [dev(x, w.dtype) for x in c["xs"]]
    wrs = [dev(x, w.dtype) for x in c["wrs"]]
    gs = [dev(x, w.dtype) for x in c["gs"]]
    wgu, wd = dev(pack_gate_up(c["wg"], c["wu"]), w.dtype), dev(c["wd"], w.dtype)
    res = []
    for recompute in (False, True):
        ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, _act(w), w.c, w.eps, w.alpha, wgrad=wgrad,
                      recompute=recompute)
        if recompute:
            assert all(st.act_a.data_ptr() == ps.layers[0].act_a.data_ptr() for st in ps.layers)
        ps.step(xs, wrs, c["sigmas"], wgu, wd, gs)
        torch.cuda.synchronize()
        res.append(ps)
    p0, p1 = res
    assert torch.equal(p0.d_w_gate_up, p1.d_w_gate_up) and torch.equal(p0.d_w_down, p1.d_w_down)
    assert torch.equal(p0.loss, p1.loss)
    for l in range(w.L):
        for field in ("out", "dx", "d_w_router", "d_sigma", "act_h", "y_perm"):
            assert torch.equal(getattr(p0.layers[l], field), getattr(p1.layers[l], field)), (l, field)


def _loop_inputs(name, n_mb):
    """n_mb micro-batches over the same weights: micro-batch m draws its tokens with seed + 100 m."""
    c = oracle_case(name)
    w = c["w"]
    batches = []
    for m in range(n_mb):
        wm = w.scaled(seed=w.seed + 100 * m)
        batches.append(([W.gen_x(wm, l) for l in range(w.L)], [W.gen_grad_out(wm, l) for l in range(w.L)]))
    return c, w, batches


@pytest.mark.parametrize("name", LOOP_CASES)
def test_lagged_loop_against_the_oracle(name):
    import torch
    from paper_2605_06665_amd.pipeline import PoolStep
    n_mb = 3
    c, w, batches = _loop_inputs(name, n_mb)
    wrs = [dev(x, w.dtype) for x in c["wrs"]]
    wgu, wd = dev(pack_gate_up(c["wg"], c["wu"]), w.dtype), dev(c["wd"], w.dtype)
    ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, _act(w), w.c, w.eps, w.alpha, lagged=True)
    tol = TOL[w.dtype]
    fbar_ref = None                     # the oracle is driven micro-batch by micro-batch with the GPU's selection
    states = []
    got = []
    for m in range(n_mb):
        xs = [dev(x, w.dtype) for x in batches[m][0]]
        gs = [dev(x, w.dtype) for x in batches[m][1]]
        states.append(ps.state_dict())
        ps.step(xs, wrs, c["sigmas"], wgu, wd, gs)
        torch.cuda.synchronize()
        idxs = []
        for l in range(w.L):
            z = O.router_logits(batches[m][0][l], c["wrs"][l])
            _, ref_idx = check_selection(z, O.topk_select(z, w.k), host(ps.layers[l].topk_idx), w.k)
            idxs.append(ref_idx)
        ref = O.pool_step(batches[m][0], c["wrs"], c["wg"], c["wu"], c["wd"], batches[m][1], w.k, c["sigmas"],
                          w.c, w.eps, w.alpha, fbar_in=fbar_ref, idxs=idxs)
        assert abs(float(host(ps.loss)[0]) - ref["loss"]) <= 1e-4 * abs(ref["loss"]), m
        assert rel_err(host(ps.aux_coef), ref["coef"]) <= 1e-5, m
        assert rel_err(host(ps.fbar), ref["fbar"]) <= 1e-6, m
        for l in range(w.L):
            assert rel_err(host(ps.layers[l].d_w_router), ref["bw"][l]["dw_router"]) <= tol, (m, l)
            assert rel_err(host(ps.layers[l].dx), ref["bw"][l]["dx"]) <= tol, (m, l)
        if m > 0:
            # the lagged coefficient is not the same-step one: the loop really used the previous statistic
            same = O.pool_aux_loss(ref["counts"], ref["psum"], w.T, w.k, w.alpha)[3]
            assert rel_err(same, ref["coef"]) > 1e-3
        fbar_ref = ref["fbar"]
        got.append([ps.loss.clone(), ps.aux_coef.clone(), ps.layers[0].d_w_router.clone(), ps.layers[0].dx.clone()])

    # checkpoint: a fresh driver that loads the state taken before micro-batch 2 repeats it bitwise
    ps2 = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, _act(w), w.c, w.eps, w.alpha, lagged=True)
    ps2.load_state_dict(states[2])
    xs = [dev(x, w.dtype) for x in batches[2][0]]
    gs = [dev(x, w.dtype) for x in batches[2][1]]
    ps2.step(xs, wrs, c["sigmas"], wgu, wd, gs)
    torch.cuda.synchronize()
    again = [ps2.loss, ps2.aux_coef, ps2.layers[0].d_w_router, ps2.layers[0].dx]
    assert all(torch.equal(a, b) for a, b in zip(got[2], again))


@pytest.mark.parametrize("name", ["C1", "bf16-tiles", "bf16-skew"])
def test_layer_aux_on_the_shared_pool(name):
    """The ablation row 'shared pool + per-layer loss' (Eq. 3 per layer, Sec. 5.4)."""
    import torch
    from paper_2605_06665_amd.pipeline import PoolStep
    c = oracle_case(name)
    w = c["w"]
    xs = [dev(x, w.dtype) for x in c["xs"]]
    wrs = [dev(x, w.dtype) for x in c["wrs"]]
    gs = [dev(x, w.dtype) for x in c["gs"]]
    wgu, wd = dev(pack_gate_up(c["wg"], c["wu"]), w.dtype), dev(c["wd"], w.dtype)
    ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, _act(w), w.c, w.eps, w.alpha, aux="layer")
    ps.step(xs, wrs, c["sigmas"], wgu, wd, gs)
    torch.cuda.synchronize()
    idxs = []
    for l in range(w.L):
        z = O.router_logits(c["xs"][l], c["wrs"][l])
        _, ref_idx = check_selection(z, O.topk_select(z, w.k), host(ps.layers[l].topk_idx), w.k)
        idxs.append(ref_idx)
    ref = O.pool_step(c["xs"], c["wrs"], c["wg"], c["wu"], c["wd"], c["gs"], w.k, c["sigmas"], w.c, w.eps,
                      w.alpha, idxs=idxs, aux="layer")
    tol = TOL[w.dtype]
    assert rel_err(host(ps.loss_layers), np.array(ref["loss_layers"])) <= 1e-4
    assert rel_err(host(ps.aux_coef_layers), ref["coef"]) <= 1e-5
    for l in range(w.L):
        assert rel_err(host(ps.layers[l].d_w_router), ref["bw"][l]["dw_router"]) <= tol, l
        assert rel_err(host(ps.layers[l].dx), ref["bw"][l]["dx"]) <= tol, l
    assert rel_err(host(ps.d_w_gate_up), np.concatenate([ref["dw_gate"], ref["dw_up"]], axis=1)) <= tol


@pytest.mark.parametrize("name", ["C1", "bf16-skew"])
def test_sharing_scope_two_groups(name):
    """G = 2 over the case's two layers: private pools, Eq. 3 per layer, no gradient across groups."""
    import torch
    from paper_2605_06665_amd.pipeline import PoolGroups
    c = oracle_case(name)
    w = c["w"]
    assert w.L == 2
    w2 = w.scaled(seed=w.seed + 1000)
    pools = [(c["wg"], c["wu"], c["wd"]), W.gen_pool_weights(w2)]
    xs = [dev(x, w.dtype) for x in c["xs"]]
    wrs = [dev(x, w.dtype) for x in c["wrs"]]
    gs = [dev(x, w.dtype) for x in c["gs"]]
    wgu = [dev(pack_gate_up(p[0], p[1]), w.dtype) for p in pools]
    wd = [dev(p[2], w.dtype) for p in pools]
    pg = PoolGroups(2, w.T, w.d, w.f, w.E, w.k, w.L, _act(w), w.c, w.eps, w.alpha)
    pg.step(xs, wrs, c["sigmas"], wgu, wd, gs)
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    groups = []
    for g in range(2):
        z = O.router_logits(c["xs"][g], c["wrs"][g])
        _, ref_idx = check_selection(z, O.topk_select(z, w.k), host(pg.groups[g].layers[0].topk_idx), w.k)
        r = O.pool_step([c["xs"][g]], [c["wrs"][g]], *pools[g], [c["gs"][g]], w.k, [c["sigmas"][g]], w.c, w.eps,
                        w.alpha, idxs=[ref_idx])
        groups.append(r)
        ps = pg.groups[g]
        assert abs(float(host(ps.loss)[0]) - r["loss"]) <= 1e-4 * abs(r["loss"])
        assert rel_err(host(ps.layers[0].d_w_router), r["bw"][0]["dw_router"]) <= tol
        assert rel_err(host(ps.layers[0].dx), r["bw"][0]["dx"]) <= tol
        assert rel_err(host(ps.d_w_gate_up), np.concatenate([r["dw_gate"], r["dw_up"]], axis=1)) <= tol
        assert rel_err(host(ps.d_w_down), r["dw_down"]) <= tol
