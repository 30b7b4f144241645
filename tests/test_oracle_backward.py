"""Pins for the oracle's backward pass: central finite differences of its own
float64 forward objective, an independent derivation by torch's autograd on a
torch-typed restatement of Eq. 2 / Eq. 7, and structural facts from App. G (pool auxiliary loss derivation)."""
import numpy as np
import pytest

from oracle import unipool_oracle as O


def problem(L=2, T=14, d=7, f=6, E=5, k=2, seed=11):
    rng = np.random.default_rng(seed)
    xs = [rng.standard_normal((T, d)) for _ in range(L)]
    wrs = [rng.standard_normal((E, d)) for _ in range(L)]
    wg = rng.standard_normal((E, f, d)) * 0.4
    wu = rng.standard_normal((E, f, d)) * 0.4
    wd = rng.standard_normal((E, d, f)) * 0.4
    gs = [rng.standard_normal((T, d)) for _ in range(L)]
    sigmas = [1.0 + 0.2 * l for l in range(L)]
    return xs, wrs, wg, wu, wd, gs, sigmas


HP = dict(k=2, c=2.3, eps=1e-6, alpha=0.05)


def _margin_ok(xs, wrs, k, tol=1e-3):
    """True if no token is within tol of a top-k switch or a ReLU kink."""
    for x, wr in zip(xs, wrs):
        z = x @ wr.T
        zs = -np.sort(-z, axis=1)
        if np.min(zs[:, k - 1] - zs[:, k]) < tol or np.min(np.abs(z)) < tol:
            return False
    return True


def _fd(fun, arr, index, h=1e-6):
    old = arr[index]
    arr[index] = old + h
    fp = fun()
    arr[index] = old - h
    fm = fun()
    arr[index] = old
    return (fp - fm) / (2 * h)


def test_all_gradients_by_central_differences():
    seed = 11
    while True:
        xs, wrs, wg, wu, wd, gs, sigmas = problem(seed=seed)
        if _margin_ok(xs, wrs, HP["k"]):
            break
        seed += 1
    step = O.pool_step(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"])
    fbar = step["fbar"].copy()                      # constant for differentiation (App. G (pool auxiliary loss derivation))

    def lam():
        return O.objective(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"],
                           HP["alpha"], fbar)

    rng = np.random.default_rng(0)

    def check(arr, grad, n=12):
        scale = np.max(np.abs(grad)) + 1e-30
        for _ in range(n):
            index = tuple(int(rng.integers(0, s)) for s in arr.shape)
            num = _fd(lam, arr, index)
            assert abs(num - grad[index]) <= 2e-7 * scale + 1e-9, (index, num, grad[index])

    for l in range(len(xs)):
        check(xs[l], step["bw"][l]["dx"])
        check(wrs[l], step["bw"][l]["dw_router"])
        # sigma is a python float: perturb through the list
        h = 1e-6
        s0 = sigmas[l]
        sigmas[l] = s0 + h
        fp = lam()
        sigmas[l] = s0 - h
        fm = lam()
        sigmas[l] = s0
        assert (fp - fm) / (2 * h) == pytest.approx(step["bw"][l]["dsigma"], rel=1e-6, abs=1e-9)
    check(wg, step["dw_gate"], 20)
    check(wu, step["dw_up"], 20)
    check(wd, step["dw_down"], 20)


def test_backward_against_autograd():
    torch = pytest.importorskip("torch")
    xs, wrs, wg, wu, wd, gs, sigmas = problem(L=3, T=20, E=6, seed=21)
    k, c, eps, alpha = 2, HP["c"], HP["eps"], HP["alpha"]
    step = O.pool_step(xs, wrs, wg, wu, wd, gs, k, sigmas, c, eps, alpha)

    def tt(a):
        return torch.tensor(np.asarray(a), dtype=torch.float64, requires_grad=True)

    txs, twrs = [tt(x) for x in xs], [tt(w) for w in wrs]
    tsig = [tt(s) for s in sigmas]
    twg, twu, twd = tt(wg), tt(wu), tt(wd)
    fbar = torch.tensor(step["fbar"])
    lam = 0.0
    pbar = 0.0
    L, T, E = len(xs), xs[0].shape[0], wg.shape[0]
    for l in range(L):
        z = txs[l] @ twrs[l].T
        s = tsig[l] * c * torch.relu(z / (torch.linalg.vector_norm(z, dim=1, keepdim=True) + eps))
        idx = torch.tensor(step["fw"][l]["idx"], dtype=torch.int64)       # selection is not differentiated
        out = torch.zeros_like(txs[l])
        for t in range(T):
            for j in range(k):
                e = int(idx[t, j])
                hid = torch.nn.functional.silu(twg[e] @ txs[l][t]) * (twu[e] @ txs[l][t])
                out[t] = out[t] + s[t, e] * (twd[e] @ hid)
        lam = lam + (out * torch.tensor(gs[l])).sum()
        pbar = pbar + s.sum(dim=0) / T / L
    lam = lam + alpha * E * (fbar * pbar).sum()
    lam.backward()
    for l in range(L):
        np.testing.assert_allclose(step["bw"][l]["dx"], txs[l].grad.numpy(), rtol=1e-9, atol=1e-11)
        np.testing.assert_allclose(step["bw"][l]["dw_router"], twrs[l].grad.numpy(), rtol=1e-9, atol=1e-11)
        assert step["bw"][l]["dsigma"] == pytest.approx(float(tsig[l].grad), rel=1e-9, abs=1e-12)
    np.testing.assert_allclose(step["dw_gate"], twg.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(step["dw_up"], twu.grad.numpy(), rtol=1e-9, atol=1e-11)
    np.testing.assert_allclose(step["dw_down"], twd.grad.numpy(), rtol=1e-9, atol=1e-11)


def test_aux_loss_reaches_only_the_router():
    # App. G (pool auxiliary loss derivation): only the routing scores carry the pool-loss gradient.
    xs, wrs, wg, wu, wd, gs, sigmas = problem(seed=4)
    zero_g = [np.zeros_like(g) for g in gs]
    step = O.pool_step(xs, wrs, wg, wu, wd, zero_g, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"])
    assert not step["dw_gate"].any() and not step["dw_up"].any() and not step["dw_down"].any()
    assert any(np.abs(bw["dw_router"]).max() > 0 for bw in step["bw"])
    assert all(not bw["dx_experts"].any() for bw in step["bw"])
    # without the aux term and without upstream gradient everything vanishes
    step0 = O.pool_step(xs, wrs, wg, wu, wd, zero_g, HP["k"], sigmas, HP["c"], HP["eps"], 0.0)
    assert all(not bw["dw_router"].any() and bw["dsigma"] == 0.0 for bw in step0["bw"])


def test_weight_grads_sum_over_layers_and_skip_idle_experts():
    xs, wrs, wg, wu, wd, gs, sigmas = problem(L=3, E=9, T=6, seed=8)     # 12 slots, 9 experts
    k, c, eps = HP["k"], HP["c"], HP["eps"]
    step = O.pool_step(xs, wrs, wg, wu, wd, gs, k, sigmas, c, eps, 0.0)
    acc = np.zeros_like(wg)
    for l in range(3):
        one = O.pool_step([xs[l]], [wrs[l]], wg, wu, wd, [gs[l]], k, [sigmas[l]], c, eps, 0.0)
        acc += one["dw_gate"]
        idle = one["counts"][0] == 0
        assert idle.any()
        assert not one["dw_gate"][idle].any() and not one["dw_down"][idle].any()
    np.testing.assert_allclose(step["dw_gate"], acc, rtol=1e-13, atol=1e-15)


def test_negative_logit_selection_has_zero_gate_and_router_gradient():
    # a selected expert with non-positive logit: counted and computed, gate 0,
    # no gradient through the ReLU
    x = np.array([[1.0, 0.0]])
    wr = np.array([[1.0, 0.0], [-1.0, 0.0], [-2.0, 0.0]])
    r = O.route(x, wr, 2, 1.0, 1.0, 0.0)
    assert r["idx"][0].tolist() == [0, 1] and r["gate"][0, 1] == 0.0
    assert r["counts"].tolist() == [1, 1, 0]
    dx, dw, dsig, dz = O.route_bwd(x, wr, r["z"], r["idx"], np.array([[0.0, 5.0]]), None, 1.0, 1.0, 0.0)
    assert not dz.any() and not dw.any() and dsig == 0.0
