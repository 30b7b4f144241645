"""Pins for the oracle's one-step-behind micro-batch loop (App. G (pool auxiliary loss derivation)) and for the recompute half of
the expert FFN (App. D (hyperparameter details)).  None of them calls the function under test to make its own expectation:
the lagged statistic is counted by hand with Python loops, the gradients come from central finite
differences of the float64 objective, the recompute is compared with a dense per-row evaluation.
The sharing-scope variants of Sec. 5.4 (per-layer loss on a shared pool, pool groups) are pinned by
a hand evaluation of Eq. 3 and finite differences."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from tests.test_oracle_backward import HP, _fd, _margin_ok, problem


def _batches(n, seed0):
    """n micro-batches that share router and pool weights; returns (batches, weights...)."""
    seed = seed0
    out = []
    base = None
    while len(out) < n:
        xs, wrs, wg, wu, wd, gs, sigmas = problem(seed=seed)
        seed += 1
        if base is None:
            base = (wrs, wg, wu, wd, sigmas)
        if _margin_ok(xs, base[0], HP["k"]):
            out.append((xs, gs))
    return out, base


def _hand_fbar(xs, wrs, k, E):
    """fbar of one micro-batch, counted slot by slot (Eq. 4): no vector code, no oracle call."""
    L = len(xs)
    fbar = [0.0] * E
    for l in range(L):
        z = xs[l] @ wrs[l].T
        T = z.shape[0]
        for t in range(T):
            order = sorted(range(E), key=lambda i: (-z[t, i], i))
            for i in order[:k]:
                fbar[i] += 1.0 / (T * k * L)
    return np.array(fbar)


def test_second_micro_batch_uses_the_first_one_s_statistic():
    batches, (wrs, wg, wu, wd, sigmas) = _batches(3, 40)
    res = O.micro_batch_loop(batches, wrs, wg, wu, wd, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"])
    E = wg.shape[0]
    L = len(wrs)
    T = batches[0][0][0].shape[0]
    for m in (1, 2):
        prev = _hand_fbar(batches[m - 1][0], wrs, HP["k"], E)
        cur = _hand_fbar(batches[m][0], wrs, HP["k"], E)
        assert np.abs(prev - cur).max() > 1e-3          # the two statistics differ: the test can tell them apart
        # loss of micro-batch m = alpha * M * sum_i fbar_i(m-1) * Pbar_i(m)        (Eq. 5 with the lagged fbar)
        pbar = np.zeros(E)
        for l in range(L):
            z = batches[m][0][l] @ wrs[l].T
            s = sigmas[l] * HP["c"] * np.maximum(z / (np.linalg.norm(z, axis=1, keepdims=True) + HP["eps"]), 0.0)
            pbar += s.mean(axis=0) / L
        assert res[m]["loss"] == pytest.approx(HP["alpha"] * E * float(prev @ pbar), rel=1e-12)
        assert np.allclose(res[m]["coef"], HP["alpha"] * E * prev / (L * T), rtol=1e-12, atol=0)
        assert np.allclose(res[m]["fbar"], cur, rtol=1e-12, atol=1e-15)     # what is handed on is the own statistic
    # the first micro-batch uses its own statistic
    own = _hand_fbar(batches[0][0], wrs, HP["k"], E)
    assert np.allclose(res[0]["coef"], HP["alpha"] * E * own / (L * T), rtol=1e-12, atol=0)


def test_lagged_gradients_by_central_differences():
    batches, (wrs, wg, wu, wd, sigmas) = _batches(2, 60)
    res = O.micro_batch_loop(batches, wrs, wg, wu, wd, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"])
    xs, gs = batches[1]
    fbar_prev = _hand_fbar(batches[0][0], wrs, HP["k"], wg.shape[0])

    def lam():
        return O.objective(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"], fbar_prev)

    rng = np.random.default_rng(3)
    for l in range(len(xs)):
        for arr, grad in ((wrs[l], res[1]["bw"][l]["dw_router"]), (xs[l], res[1]["bw"][l]["dx"])):
            scale = np.max(np.abs(grad)) + 1e-30
            for _ in range(10):
                index = tuple(int(rng.integers(0, n)) for n in arr.shape)
                num = _fd(lam, arr, index)
                assert abs(num - grad[index]) <= 2e-7 * scale + 1e-9, (l, index, num, grad[index])


def test_lagged_equals_same_step_when_the_batches_repeat():
    batches, (wrs, wg, wu, wd, sigmas) = _batches(1, 80)
    twice = [batches[0], batches[0]]
    res = O.micro_batch_loop(twice, wrs, wg, wu, wd, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"])
    assert res[1]["loss"] == pytest.approx(res[0]["loss"], rel=1e-14)
    for l in range(len(wrs)):
        assert np.array_equal(res[1]["bw"][l]["dw_router"], res[0]["bw"][l]["dw_router"])


def test_given_initial_statistic_is_used_as_is():
    batches, (wrs, wg, wu, wd, sigmas) = _batches(1, 90)
    E = wg.shape[0]
    f0 = np.full(E, 1.0 / E)
    res = O.micro_batch_loop(batches, wrs, wg, wu, wd, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"], fbar0=f0)
    L, T = len(wrs), batches[0][0][0].shape[0]
    # uniform fbar: every expert's coefficient is alpha / (L T)
    assert np.allclose(res[0]["coef"], HP["alpha"] / (L * T), rtol=1e-12, atol=0)


def test_recompute_matches_dense_rows():
    rng = np.random.default_rng(5)
    E, f, d, S = 4, 5, 6, 17
    wg = rng.standard_normal((E, f, d))
    wu = rng.standard_normal((E, f, d))
    x = rng.standard_normal((S, d))
    offsets = np.array([0, 6, 6, 13, 17])            # expert 1 has no rows
    a, b, h = O.expert_ffn_recompute(x, offsets, wg, wu)
    for row in range(S):
        e = int(np.searchsorted(offsets, row, side="right") - 1)
        for n in range(f):
            aa = sum(x[row, c] * wg[e, n, c] for c in range(d))
            bb = sum(x[row, c] * wu[e, n, c] for c in range(d))
            assert a[row, n] == pytest.approx(aa, rel=1e-12, abs=1e-14)
            assert b[row, n] == pytest.approx(bb, rel=1e-12, abs=1e-14)
            assert h[row, n] == pytest.approx(aa / (1.0 + np.exp(-aa)) * bb, rel=1e-12, abs=1e-14)


# --------------------------------------------------------------------------- sharing scope, layer aux
def _hand_layer_loss(x, wr, sigma, k, E):
    """Eq. 3 for one layer with Python loops: alpha-free  E * sum_i f_i P_i."""
    z = x @ wr.T
    T = z.shape[0]
    f = [0.0] * E
    P = [0.0] * E
    for t in range(T):
        order = sorted(range(E), key=lambda i: (-z[t, i], i))
        for i in order[:k]:
            f[i] += 1.0 / (T * k)
        nrm = float(np.sqrt(sum(z[t, i] ** 2 for i in range(E)))) + HP["eps"]
        for i in range(E):
            P[i] += sigma * HP["c"] * max(z[t, i] / nrm, 0.0) / T
    return E * sum(fi * pi for fi, pi in zip(f, P)), np.array(f)


def test_layer_aux_on_a_shared_pool():
    batches, (wrs, wg, wu, wd, sigmas) = _batches(1, 120)
    xs, gs = batches[0]
    E, L, T = wg.shape[0], len(wrs), xs[0].shape[0]
    res = O.pool_step(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"], aux="layer")
    total = 0.0
    for l in range(L):
        hand, f = _hand_layer_loss(xs[l], wrs[l], sigmas[l], HP["k"], E)
        assert res["loss_layers"][l] == pytest.approx(HP["alpha"] * hand, rel=1e-12)
        assert np.allclose(res["coef"][l], HP["alpha"] * E * f / T, rtol=1e-12, atol=0)
        total += HP["alpha"] * hand
    assert res["loss"] == pytest.approx(total, rel=1e-12)
    # gradient of the summed per-layer losses, f^(l) held constant, by central differences
    fl = [res["fbar"][l].copy() for l in range(L)]

    def lam():
        tot = 0.0
        for l in range(L):
            fw = O.moe_layer_fwd(xs[l], wrs[l], wg, wu, wd, HP["k"], sigmas[l], HP["c"], HP["eps"])
            tot += float(np.sum(fw["out"] * gs[l])) + HP["alpha"] * E * float(np.sum(fl[l] * fw["psum"] / T))
        return tot

    rng = np.random.default_rng(9)
    for l in range(L):
        grad = res["bw"][l]["dw_router"]
        scale = np.max(np.abs(grad))
        for _ in range(10):
            index = tuple(int(rng.integers(0, n)) for n in wrs[l].shape)
            num = _fd(lam, wrs[l], index)
            assert abs(num - grad[index]) <= 2e-7 * scale + 1e-9


def test_sharing_scope_groups():
    (xs, gs), = _batches(1, 140)[0]
    _, (wrs, wg, wu, wd, sigmas) = _batches(1, 140)
    L = len(wrs)
    # G = 1: the group step is the pool step
    one = dict(xs=xs, w_routers=wrs, w_gate=wg, w_up=wu, w_down=wd, grad_outs=gs, sigmas=sigmas)
    res, total = O.pool_groups_step([one], HP["k"], HP["c"], HP["eps"], HP["alpha"])
    ref = O.pool_step(xs, wrs, wg, wu, wd, gs, HP["k"], sigmas, HP["c"], HP["eps"], HP["alpha"])
    assert total == ref["loss"] and np.array_equal(res[0]["dw_gate"], ref["dw_gate"])
    # one layer per group, private pools: Eq. 3 per layer, and no gradient crosses the groups
    rng = np.random.default_rng(1)
    pools = [(wg, wu, wd)] + [tuple(rng.standard_normal(w.shape) * 0.4 for w in (wg, wu, wd)) for _ in range(L - 1)]
    groups = [dict(xs=[xs[l]], w_routers=[wrs[l]], w_gate=pools[l][0], w_up=pools[l][1], w_down=pools[l][2],
                   grad_outs=[gs[l]], sigmas=[sigmas[l]]) for l in range(L)]
    res, total = O.pool_groups_step(groups, HP["k"], HP["c"], HP["eps"], HP["alpha"])
    E = wg.shape[0]
    hand_total = 0.0
    for l in range(L):
        hand, _ = _hand_layer_loss(xs[l], wrs[l], sigmas[l], HP["k"], E)
        assert res[l]["loss"] == pytest.approx(HP["alpha"] * hand, rel=1e-12)
        hand_total += HP["alpha"] * hand
        # a private pool's weight gradient is that of a dense sum over this layer's tokens only
        out = O.moe_layer_fwd(xs[l], wrs[l], *pools[l], HP["k"], sigmas[l], HP["c"], HP["eps"])
        assert np.array_equal(out["counts"], res[l]["counts"][0])
    assert total == pytest.approx(hand_total, rel=1e-12)
