"""GPU parity of the softmax router kind (the comparison router of Sec. 5.4) behind the same entry points:
unipool_route and unipool_route_bwd element by element against the oracle, and whole steps."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
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


def test_unknown_router_kind_is_rejected():
    U = lib()
    sh = shape_of(CASES["C1"])
    sh.router = 5
    with pytest.raises(U.UniPoolError, match="router 5"):
        U.workspace_bytes(sh)
