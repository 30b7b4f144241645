"""GPU parity on the degenerate inputs of the method: a token whose logits are all zero (norm 0, only
epsilon in the denominator of Eq. 7) and a layer in which one expert takes every slot while all the
others stay empty."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import TOL, check_selection, dev, host, rel_err
from tests.test_gpu_parity import empty, lib, pack_gate_up, shape_of, workspace

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_zero_token(dtype):
    """x_t = 0 gives z = 0: scores and gates 0, exact ties resolved to the lowest indices, no gradient
    through the normalisation (and no NaN anywhere)."""
    import torch
    w = W.Workload("zero-token-" + dtype, L=1, E=16, d=64, f=64, k=3, T=130, dtype=dtype, seed=51, c=2.2)
    U = lib()
    sh = shape_of(w)
    x_h, wr_h = W.gen_x(w, 0), W.gen_w_router(w, 0)
    zero_rows = [0, 77, 129]
    x_h[zero_rows] = 0.0
    ref = O.route(x_h, wr_h, w.k, w.sigma, w.c, w.eps)
    assert ref["idx"][zero_rows].tolist() == [[0, 1, 2]] * 3 and not ref["gate"][zero_rows].any()
    x, wr = dev(x_h, dtype), dev(wr_h, dtype)
    idx, gate = empty((w.T, w.k), "i32"), empty((w.T, w.k), "f32")
    logits, counts, psum = empty((w.T, w.E), "f32"), empty((w.E,), "i32"), empty((w.E,), "f32")
    ws = workspace(sh)
    U.route(sh, x, wr, idx, gate, logits, counts, psum, ws)
    torch.cuda.synchronize()
    tol = TOL[dtype]
    gi = host(idx)
    assert gi[zero_rows].tolist() == [[0, 1, 2]] * 3, "exact ties go to the lower index"
    assert not host(gate)[zero_rows].any() and not host(logits)[zero_rows].any()
    check_selection(ref["z"], ref["idx"], gi, w.k, scores=ref["s"], got_gate=host(gate), tol=tol)
    assert np.array_equal(host(counts), np.bincount(gi.ravel(), minlength=w.E))
    assert rel_err(host(psum), ref["psum"]) <= tol
    # backward: the zero tokens contribute nothing and nothing becomes NaN
    rng = np.random.default_rng(1)
    dgate = rng.standard_normal((w.T, w.k)).astype(np.float32)
    coef = (rng.random(w.E) * 1e-3).astype(np.float32)
    z32 = ref["z"].astype(np.float32)
    dx, dw, dsig, dz = O.route_bwd(x_h, wr_h, z32, gi, dgate, coef, w.sigma, w.c, w.eps)
    assert not dx[zero_rows].any()
    g_dx, g_dw, g_ds = empty((w.T, w.d), dtype), empty((w.E, w.d), "f32"), empty((1,), "f32")
    U.route_bwd(sh, x, wr, dev(z32), dev(gi.astype(np.int32)), dev(dgate), dev(coef), g_dw, g_ds, g_dx, False, ws)
    torch.cuda.synchronize()
    assert np.isfinite(host(g_dx)).all() and np.isfinite(host(g_dw)).all()
    assert not host(g_dx)[zero_rows].any()
    assert rel_err(host(g_dx), dx) <= tol and rel_err(host(g_dw), dw) <= tol
    assert abs(float(host(g_ds)[0]) - dsig) <= tol * max(abs(dsig), 1e-3)


@pytest.mark.parametrize("wgrad", ["pool", "layer"])
def test_one_expert_takes_every_slot(wgrad):
    """Top-1 routing with one expert's logit far above the rest: that expert holds all T rows (several
    row tiles), every other expert is empty in that layer; the second layer routes normally."""
    import torch
    from paper_2605_06665_amd.pipeline import PoolStep
    w = W.Workload("one-expert", L=2, E=8, d=128, f=192, k=1, T=700, dtype="bf16", seed=52, c=1.9)
    U = lib()
    xs = [W.gen_x(w, l) for l in range(w.L)]
    wrs = [W.gen_w_router(w, l) for l in range(w.L)]
    gs = [W.gen_grad_out(w, l) for l in range(w.L)]
    wg, wu, wd = W.gen_pool_weights(w)
    xs[0][:, w.d - 1] = 1.0                      # a constant feature ...
    wrs[0][:, w.d - 1] = 0.0
    wrs[0][5, w.d - 1] = 256.0                   # ... that lifts expert 5's logit above every other one
    sig = [1.0, 1.2]
    ps = PoolStep(w.T, w.d, w.f, w.E, w.k, w.L, U.BF16, w.c, w.eps, w.alpha, wgrad=wgrad)
    dx = [dev(x, "bf16") for x in xs]
    ps.step(dx, [dev(x, "bf16") for x in wrs], sig, dev(pack_gate_up(wg, wu), "bf16"), dev(wd, "bf16"),
            [dev(g, "bf16") for g in gs])
    torch.cuda.synchronize()
    c0 = host(ps.counts[0])
    assert c0[5] == w.T and c0.sum() == w.T, "expert 5 holds every slot of layer 0"
    idxs = []
    for l in range(w.L):
        z = O.router_logits(xs[l], wrs[l])
        _, merged = check_selection(z, O.topk_select(z, w.k), host(ps.layers[l].topk_idx), w.k)
        idxs.append(merged)
    ref = O.pool_step(xs, wrs, wg, wu, wd, gs, w.k, sig, w.c, w.eps, w.alpha, idxs=idxs)
    tol = TOL["bf16"]
    assert np.array_equal(host(ps.counts), ref["counts"])
    assert abs(float(host(ps.loss)[0]) - ref["loss"]) <= 1e-4 * abs(ref["loss"])
    for l in range(w.L):
        st, fw, bw = ps.layers[l], ref["fw"][l], ref["bw"][l]
        assert np.array_equal(host(st.offsets), fw["offsets"])
        assert np.array_equal(host(st.row_of_slot), fw["row_of_slot"])
        assert rel_err(host(st.out), fw["out"]) <= tol
        assert rel_err(host(st.dx), bw["dx"]) <= tol
        assert rel_err(host(st.d_w_router), bw["dw_router"]) <= tol
    assert rel_err(host(ps.d_w_gate_up), np.concatenate([ref["dw_gate"], ref["dw_up"]], axis=1)) <= tol
    assert rel_err(host(ps.d_w_down), ref["dw_down"]) <= tol
