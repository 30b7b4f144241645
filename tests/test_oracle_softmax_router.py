"""Pins of the oracle's softmax router (the comparison router of Sec. 5.4; Eq. 1 and Eq. 3 use softmax
probabilities): rows sum to one, a hand example, shift invariance, the pool loss equal to alpha under exactly
uniform usage (closed form: sum_i (1/M) * Pbar_i * M * alpha with sum_i Pbar_i = 1), agreement with an
independent softmax (scipy), and every gradient by central finite differences and by torch autograd."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from tests.test_oracle_backward import HP, _fd, _margin_ok, problem


def test_hand_example_and_rows_sum_to_one():
    z = np.array([[0.0, np.log(2.0), np.log(5.0)], [1.0, 1.0, 1.0]])
    p = O.softmax_router_scores(z)
    assert np.allclose(p[0], [1 / 8, 2 / 8, 5 / 8], atol=1e-15)
    assert np.allclose(p[1], [1 / 3] * 3, atol=1e-15)
    rng = np.random.default_rng(1)
    z = rng.standard_normal((50, 17)) * 30.0                      # large logits: no overflow
    p = O.softmax_router_scores(z)
    assert np.all(np.isfinite(p)) and np.allclose(p.sum(axis=1), 1.0, atol=1e-14)
    assert np.allclose(O.softmax_router_scores(z + 123.0), p, atol=1e-12)      # shift invariance
    from scipy.special import softmax
    assert np.allclose(p, softmax(z, axis=1), atol=1e-15)


def test_gates_and_statistics():
    rng = np.random.default_rng(2)
    x, wr = rng.standard_normal((40, 9)), rng.standard_normal((6, 9))
    r = O.route(x, wr, 2, 1.0, 2.0, 1e-6, router="softmax")
    z = x @ wr.T
    for t in range(40):                                           # by counting, token by token
        e = np.exp(z[t] - z[t].max())
        p = e / e.sum()
        order = sorted(range(6), key=lambda i: (-z[t, i], i))[:2]
        assert r["idx"][t].tolist() == order
        assert np.allclose(r["gate"][t], p[order], atol=1e-14)
    assert np.isclose(r["psum"].sum(), 40.0, atol=1e-10)          # probabilities: every token adds one
    # sigma, c and eps play no part
    r2 = O.route(x, wr, 2, 3.0, 7.0, 0.5, router="softmax")
    assert np.array_equal(r["gate"], r2["gate"])


def test_pool_loss_is_alpha_under_exactly_uniform_usage():
    L, E, T, k, alpha = 3, 8, 16, 2, 0.02
    rng = np.random.default_rng(3)
    counts = np.full((L, E), T * k // E)                          # every expert gets the same share
    psum = np.stack([O.softmax_router_scores(rng.standard_normal((T, E))).sum(axis=0) for _ in range(L)])
    _, fbar, loss, _ = O.pool_aux_loss(counts, psum, T, k, alpha)
    assert np.allclose(fbar, 1.0 / E)
    assert np.isclose(loss, alpha, rtol=1e-13)


def test_gradients_by_central_differences():
    seed = 21
    while True:
        xs, wrs, wg, wu, wd, gs, sigmas = problem(seed=seed)
        if _margin_ok(xs, wrs, HP["k"]):
            break
        seed += 1
    step = O.pool_step(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"],
                       router="softmax")
    fbar = step["fbar"].copy()

    def lam():
        return O.objective(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"], fbar,
                           router="softmax")
    rng = np.random.default_rng(0)
    for l in range(len(xs)):
        for _ in range(6):
            i = (int(rng.integers(xs[l].shape[0])), int(rng.integers(xs[l].shape[1])))
            assert np.isclose(_fd(lam, xs[l], i), step["bw"][l]["dx"][i], rtol=2e-6, atol=1e-8)
            j = (int(rng.integers(wrs[l].shape[0])), int(rng.integers(wrs[l].shape[1])))
            assert np.isclose(_fd(lam, wrs[l], j), step["bw"][l]["dw_router"][j], rtol=2e-6, atol=1e-8)
        assert step["bw"][l]["dsigma"] == 0.0
    for arr, grad in ((wg, step["dw_gate"]), (wu, step["dw_up"]), (wd, step["dw_down"])):
        for _ in range(6):
            i = tuple(int(rng.integers(n)) for n in arr.shape)
            assert np.isclose(_fd(lam, arr, i), grad[i], rtol=2e-6, atol=1e-8)


def test_router_backward_against_autograd():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(5)
    T, d, E, k = 12, 6, 7, 3
    x, wr = rng.standard_normal((T, d)), rng.standard_normal((E, d))
    r = O.route(x, wr, k, 1.0, 1.0, 0.0, router="softmax")
    dgate = rng.standard_normal((T, k))
    coef = rng.random(E) * 0.1
    dx, dw, dsig, dz = O.route_bwd(x, wr, r["z"], r["idx"], dgate, coef, 1.0, 1.0, 0.0, router="softmax")
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tw = torch.tensor(wr, dtype=torch.float64, requires_grad=True)
    p = torch.softmax(tx @ tw.T, dim=1)
    picked = torch.gather(p, 1, torch.tensor(r["idx"].astype(np.int64)))
    obj = (picked * torch.tensor(dgate)).sum() + (p * torch.tensor(coef)[None, :]).sum()
    obj.backward()
    assert np.allclose(tx.grad.numpy(), dx, atol=1e-12) and np.allclose(tw.grad.numpy(), dw, atol=1e-12)
    assert dsig == 0.0 and np.allclose(dz.sum(axis=1), 0.0, atol=1e-13)      # softmax gradients sum to zero


def test_vanilla_moe_is_one_layer_per_group_with_the_softmax_router():
    """The comparison system of Eq. 1 / Eq. 3: private experts per layer, top-1 softmax router, per-layer loss.
    Its loss is alpha E sum_i f_i P_i by hand for every layer, its output the selected expert's output times
    the selected probability, and no weight gradient crosses the layers."""
    rng = np.random.default_rng(7)
    L, T, d, f, E = 3, 60, 10, 12, 5
    xs = [rng.standard_normal((T, d)) for _ in range(L)]
    gs = [rng.standard_normal((T, d)) for _ in range(L)]
    wrs = [rng.standard_normal((E, d)) for _ in range(L)]
    pools = [tuple(rng.standard_normal(s) * 0.3 for s in ((E, f, d), (E, f, d), (E, d, f))) for _ in range(L)]
    alpha = 0.02
    groups = [dict(xs=[xs[l]], w_routers=[wrs[l]], w_gate=pools[l][0], w_up=pools[l][1], w_down=pools[l][2],
                   grad_outs=[gs[l]], sigmas=[1.0]) for l in range(L)]
    res, total = O.pool_groups_step(groups, 1, 1.0, 1e-6, alpha, router="softmax")
    hand_total = 0.0
    for l in range(L):
        z = xs[l] @ wrs[l].T
        p = np.exp(z - z.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        sel = np.argmax(z, axis=1)
        fvec = np.bincount(sel, minlength=E) / T
        hand = alpha * E * float(np.sum(fvec * p.mean(axis=0)))
        assert res[l]["loss"] == pytest.approx(hand, rel=1e-12)
        hand_total += hand
        # token 0 by hand: the selected expert's SwiGLU output times its probability
        e = sel[0]
        a, b = pools[l][0][e] @ xs[l][0], pools[l][1][e] @ xs[l][0]
        y = pools[l][2][e] @ (a / (1.0 + np.exp(-a)) * b)
        assert np.allclose(res[l]["fw"][0]["out"][0], p[0, e] * y, atol=1e-12)
        # experts that no token of this layer selected get no gradient
        idle = np.setdiff1d(np.arange(E), sel)
        assert not np.any(res[l]["dw_down"][idle])
    assert total == pytest.approx(hand_total, rel=1e-12)
