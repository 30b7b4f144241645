"""GPU parity of the softmax router kind (the comparison router of Sec. 5.4) behind the same entry points:
unipool_route and unipool_route_bwd element by element against the oracle, and whole steps."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import TOL, check_selection, dev, host, rel_err, round_act
from tests.test_gpu_parity import CASES, empty, lib, oracle_case, pack_gate_up, shape_of, workspace

pytestmark = pytest.mark.gpu

# float mode, fused bfloat16 router (E <= 256), pool beyond the fused router, skewed routing, k = E
NAMES = ["C1", "f32-ragged", "bf16-tiles", "bf16-skew", "bf16-k8", "bf16-kE", "bf16-fewtok-bigE"]


def _shape(w, sigma=None):
    sh = shape_of(w, sigma)
    sh.router = lib().ROUTER_SOFTMAX
    return sh


@pytest.mark.parametrize("name", NAMES)
def test_route_softmax(name):
    import torch
    c = oracle_case(name)
    w, U = c["w"], lib()
    sh = _shape(w)
    ref = O.route(c["xs"][0], c["wrs"][0], w.k, w.sigma, w.c, w.eps, router="softmax")
    x, wr = dev(c["xs"][0], w.dtype), dev(c["wrs"][0], w.dtype)
    idx, gate = empty((w.T, w.k), "i32"), empty((w.T, w.k), "f32")
    logits, counts, psum = empty((w.T, w.E), "f32"), empty((w.E,), "i32"), empty((w.E,), "f32")
    U.route(sh, x, wr, idx, gate, logits, counts, psum, workspace(sh))
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    assert rel_err(host(logits), ref["z"]) <= tol
    gi = host(idx)
    check_selection(ref["z"], ref["idx"], gi, w.k, scores=ref["s"], got_gate=host(gate), tol=tol)
    assert np.array_equal(host(counts), np.bincount(gi.ravel(), minlength=w.E))
    assert rel_err(host(psum), ref["psum"]) <= tol
    assert abs(float(host(psum).sum()) - w.T) <= tol * w.T          # probabilities: every token adds one


@pytest.mark.parametrize("name", NAMES)
def test_route_bwd_softmax(name):
    import torch
    c = oracle_case(name)
    w, U = c["w"], lib()
    sh = _shape(w)
    r = O.route(c["xs"][0], c["wrs"][0], w.k, w.sigma, w.c, w.eps, router="softmax")
    rng = np.random.default_rng(8)
    dgate = rng.standard_normal((w.T, w.k)).astype(np.float32)
    coef = (rng.random(w.E) * 1e-2).astype(np.float32)
    z32 = r["z"].astype(np.float32)
    dx, dw, dsig, dz = O.route_bwd(c["xs"][0], c["wrs"][0], z32, r["idx"], dgate, coef, w.sigma, w.c, w.eps,
                                   router="softmax")
    g_dx, g_dw, g_ds = empty((w.T, w.d), w.dtype), empty((w.E, w.d), "f32"), empty((1,), "f32")
    U.route_bwd(sh, dev(c["xs"][0], w.dtype), dev(c["wrs"][0], w.dtype), dev(z32), dev(r["idx"].astype(np.int32)),
                dev(dgate), dev(coef), g_dw, g_ds, g_dx, False, workspace(sh))
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    assert rel_err(host(g_dw), dw) <= tol
    assert rel_err(host(g_dx), dx) <= tol
    assert float(host(g_ds)[0]) == 0.0 and dsig == 0.0


@pytest.mark.parametrize("name", ["C1", "bf16-tiles", "bf16-skew"])
def test_whole_step_softmax(name):
    import torch
    from paper_2605_06665_amd.pipeline import PoolStep
    c = oracle_case(name)
    w, U = c["w"], lib()
    ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, U.BF16 if w.dtype == "bf16" else U.F32, w.c, w.eps, w.alpha,
                  router="softmax")
    xs = [dev(x, w.dtype) for x in c["xs"]]
    wrs = [dev(x, w.dtype) for x in c["wrs"]]
    gs = [dev(x, w.dtype) for x in c["gs"]]
    ps.step(xs, wrs, c["sigmas"], dev(pack_gate_up(c["wg"], c["wu"]), w.dtype), dev(c["wd"], w.dtype), gs)
    torch.cuda.synchronize()
    idxs = []
    for l in range(w.L):
        z = O.router_logits(c["xs"][l], c["wrs"][l])
        _, merged = check_selection(z, O.topk_select(z, w.k), host(ps.layers[l].topk_idx), w.k)
        idxs.append(merged)
    ref = O.pool_step(c["xs"], c["wrs"], c["wg"], c["wu"], c["wd"], c["gs"], w.k, c["sigmas"], w.c, w.eps,
                      w.alpha, idxs=idxs, router="softmax")
    tol = TOL[w.dtype]
    assert np.array_equal(host(ps.counts), ref["counts"])
    assert abs(float(host(ps.loss)[0]) - ref["loss"]) <= 1e-4 * abs(ref["loss"])
    for l in range(w.L):
        st, fw, bw = ps.layers[l], ref["fw"][l], ref["bw"][l]
        assert rel_err(host(st.out), fw["out"]) <= tol, "out"
        assert rel_err(host(st.dx), bw["dx"]) <= tol, "dx"
        assert rel_err(host(st.d_w_router), bw["dw_router"]) <= tol, "dw_router"
    assert rel_err(host(ps.d_w_gate_up), np.concatenate([ref["dw_gate"], ref["dw_up"]], axis=1)) <= tol
    assert rel_err(host(ps.d_w_down), ref["dw_down"]) <= tol


VANILLA = {
    "f32": W.Workload("vanilla-f32", L=3, E=8, d=48, f=40, k=1, T=210, dtype="f32", seed=71, c=1.0),
    "bf16": W.Workload("vanilla-bf16", L=4, E=8, d=128, f=192, k=1, T=1500, dtype="bf16", seed=72, c=1.0),
}


@pytest.mark.parametrize("kind", list(VANILLA))
def test_vanilla_moe_layer_private_experts_top1_softmax(kind):
    """The comparison system of the paper (Eq. 1, Eq. 3; 8 experts per layer, top-1, softmax router): one group
    per layer, each with experts, loss and weight gradient of its own, through the same entry points."""
    import torch
    from paper_2605_06665_amd.pipeline import PoolGroups
    w, U = VANILLA[kind], lib()
    xs = [W.gen_x(w, l) for l in range(w.L)]
    wrs = [W.gen_w_router(w, l) for l in range(w.L)]
    gs = [W.gen_grad_out(w, l) for l in range(w.L)]
    pools = [W.gen_pool_weights(w.scaled(seed=w.seed + 100 * l)) for l in range(w.L)]
    sigmas = [1.0] * w.L
    pg = PoolGroups(w.L, w.T, w.d, w.f, w.E, w.k, w.L, U.BF16 if w.dtype == "bf16" else U.F32, w.c, w.eps, w.alpha,
                    router="softmax")
    pg.step([dev(x, w.dtype) for x in xs], [dev(x, w.dtype) for x in wrs], sigmas,
            [dev(pack_gate_up(p[0], p[1]), w.dtype) for p in pools], [dev(p[2], w.dtype) for p in pools],
            [dev(x, w.dtype) for x in gs])
    torch.cuda.synchronize()
    tol = TOL[w.dtype]
    total = 0.0
    for l in range(w.L):
        ps = pg.groups[l]
        z = O.router_logits(xs[l], wrs[l])
        _, merged = check_selection(z, O.topk_select(z, w.k), host(ps.layers[0].topk_idx), w.k)
        ref = O.pool_step([xs[l]], [wrs[l]], *pools[l], [gs[l]], w.k, [1.0], w.c, w.eps, w.alpha, idxs=[merged],
                          router="softmax")
        total += ref["loss"]
        assert np.array_equal(host(ps.counts), ref["counts"])
        assert abs(float(host(ps.loss)[0]) - ref["loss"]) <= 1e-4 * abs(ref["loss"])
        assert rel_err(host(ps.layers[0].out), ref["fw"][0]["out"]) <= tol
        assert rel_err(host(ps.layers[0].dx), ref["bw"][0]["dx"]) <= tol
        assert rel_err(host(ps.layers[0].d_w_router), ref["bw"][0]["dw_router"]) <= tol
        assert rel_err(host(ps.d_w_gate_up), np.concatenate([ref["dw_gate"], ref["dw_up"]], axis=1)) <= tol
        assert rel_err(host(ps.d_w_down), ref["dw_down"]) <= tol
    # the same groups through the oracle's own group step give the same total
    if all(np.array_equal(host(pg.groups[l].layers[0].topk_idx).ravel(),
                          np.argmax(O.router_logits(xs[l], wrs[l]), axis=1)) for l in range(w.L)):
        groups = [dict(xs=[xs[l]], w_routers=[wrs[l]], w_gate=pools[l][0], w_up=pools[l][1], w_down=pools[l][2],
                       grad_outs=[gs[l]], sigmas=[1.0]) for l in range(w.L)]
        _, ref_total = O.pool_groups_step(groups, w.k, w.c, w.eps, w.alpha, router="softmax")
        assert abs(ref_total - total) <= 1e-12 * abs(total)


def test_unknown_router_kind_is_rejected():
    U = lib()
    sh = shape_of(CASES["C1"])
    sh.router = 5
    with pytest.raises(U.UniPoolError, match="router 5"):
        U.workspace_bytes(sh)
