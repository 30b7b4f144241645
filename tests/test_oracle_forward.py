"""Pins for the oracle's forward pass: things the paper and mathematics fix,
none of which call the oracle's own routines to produce the expected value."""
import json
import math
import os

import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny(T=24, d=10, f=12, E=6, k=2, seed=3, wstd=0.3):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, d))
    wr = rng.standard_normal((E, d))
    wg = rng.standard_normal((E, f, d)) * wstd
    wu = rng.standard_normal((E, f, d)) * wstd
    wd = rng.standard_normal((E, d, f)) * wstd
    return x, wr, wg, wu, wd


# ------------------------------------------------------------------ Eq. 7
def test_normrouter_hand_values():
    g = json.load(open(os.path.join(GOLDEN, "normrouter_hand_example.json")))
    a = g["normrouter"]
    s, n = O.norm_router_scores(np.array([a["z"]]), a["sigma"], a["c"], a["eps"])
    assert n[0] == pytest.approx(a["norm"], abs=1e-15)
    np.testing.assert_allclose(s[0], a["s"], atol=1e-15)
    idx = O.topk_select(np.array([a["z"]]), 2)
    assert idx[0].tolist() == a["top2"]          # tie between the two zeros -> lower index
    b = g["normrouter_eps"]
    s, _ = O.norm_router_scores(np.array([b["z"]]), b["sigma"], b["c"], b["eps"])
    np.testing.assert_allclose(s[0], b["s"], atol=1e-15)   # eps sits outside the norm


def test_normrouter_invariants():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((4000, 96))
    sigma, c, eps = 1.3, 3.0, 1e-6
    s, n = O.norm_router_scores(z, sigma, c, eps)
    # bounded magnitude: sum s^2 <= (sigma c)^2, with equality iff no negative logits
    assert np.all(np.sum(s * s, axis=1) <= (sigma * c) ** 2 + 1e-12)
    # zhat has norm n/(n+eps): recover it from positive and negative parts
    sneg, _ = O.norm_router_scores(-z, sigma, c, eps)
    total = (np.sum(s * s, axis=1) + np.sum(sneg * sneg, axis=1)) / (sigma * c) ** 2
    np.testing.assert_allclose(total, (n / (n + eps)) ** 2, rtol=1e-12)
    # about half of the experts get a zero score on Gaussian logits (Sec. 4.3)
    assert abs(np.mean(s == 0.0) - 0.5) < 0.01
    # scale invariance of the direction: scores of lambda*z equal scores of z up to eps/n
    s2, _ = O.norm_router_scores(37.0 * z, sigma, c, eps)
    np.testing.assert_allclose(s2, s, rtol=1e-6, atol=1e-9)


def test_topk_against_full_sort_with_ties():
    rng = np.random.default_rng(1)
    # small integer logits force many exact ties, including all-negative rows
    z = rng.integers(-3, 3, size=(500, 7)).astype(np.float64)
    z[0] = -1.0
    z[1] = 0.0
    for k in (1, 2, 3, 7):
        idx = O.topk_select(z, k)
        for t in range(z.shape[0]):
            ranked = sorted(range(7), key=lambda i: (-z[t, i], i))   # python's own stable sort
            assert idx[t].tolist() == ranked[:k]


def test_route_statistics_by_counting():
    x, wr, *_ = tiny(T=50, E=9, k=3)
    r = O.route(x, wr, 3, 1.0, 2.0, 1e-6)
    T, E = 50, 9
    counts = [0] * E
    psum = [0.0] * E
    for t in range(T):
        z = [sum(wr[i, c_] * x[t, c_] for c_ in range(x.shape[1])) for i in range(E)]
        n = math.sqrt(sum(v * v for v in z))
        s = [2.0 * max(0.0, v / (n + 1e-6)) for v in z]
        top = sorted(range(E), key=lambda i: (-z[i], i))[:3]
        assert r["idx"][t].tolist() == top
        for j, i in enumerate(top):
            counts[i] += 1
            assert r["gate"][t, j] == pytest.approx(s[i], rel=1e-12, abs=1e-15)
        for i in range(E):
            psum[i] += s[i]
    assert r["counts"].tolist() == counts
    np.testing.assert_allclose(r["psum"], psum, rtol=1e-12)
    assert int(r["counts"].sum()) == T * 3


# ------------------------------------------------------------------ permutation
@pytest.mark.parametrize("T,E,k", [(1, 1, 1), (17, 5, 2), (64, 8, 8), (100, 33, 4)])
def test_permutation_invariants(T, E, k):
    rng = np.random.default_rng(T * 100 + E)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    off, ros, sor = O.permutation(idx, E)
    S = T * k
    assert off[0] == 0 and off[E] == S and np.all(np.diff(off) >= 0)
    assert sorted(ros.ravel().tolist()) == list(range(S))            # bijection
    assert np.array_equal(sor[ros.ravel()], np.arange(S))            # inverse pair
    for e in range(E):
        slots = sor[off[e]:off[e + 1]]
        assert np.all(idx.ravel()[slots] == e)                       # group holds only expert e
        toks = slots // k
        assert np.all(np.diff(toks) > 0)                             # ascending tokens
        assert off[e + 1] - off[e] == int(np.sum(idx == e))
    x = rng.standard_normal((T, 3))
    xp = O.permute_rows(x, sor, k)
    for t in range(T):
        for j in range(k):
            assert np.array_equal(xp[ros[t, j]], x[t])


def test_permutation_empty_experts():
    idx = np.array([[2], [2], [5]], dtype=np.int32)
    off, ros, sor = O.permutation(idx, 7)
    assert off.tolist() == [0, 0, 0, 2, 2, 2, 3, 3]
    assert ros.ravel().tolist() == [0, 1, 2]


# ------------------------------------------------------------------ Eq. 2 by brute force
def _py_silu(v):
    return v / (1.0 + math.exp(-v))


def _dense_expert(xt, wg, wu, wd):
    f, d = wg.shape
    h = []
    for n in range(f):
        a = sum(wg[n, c_] * xt[c_] for c_ in range(d))
        b = sum(wu[n, c_] * xt[c_] for c_ in range(d))
        h.append(_py_silu(a) * b)
    return [sum(wd[m, n] * h[n] for n in range(f)) for m in range(wd.shape[0])]


@pytest.mark.parametrize("k", [1, 2, 6])
def test_sparse_layer_equals_dense_masked_sum(k):
    x, wr, wg, wu, wd = tiny(T=10, d=6, f=7, E=6, k=k)
    sigma, c, eps = 0.8, 2.2, 1e-6
    fw = O.moe_layer_fwd(x, wr, wg, wu, wd, k, sigma, c, eps)
    T, d = x.shape
    E = wr.shape[0]
    for t in range(T):
        z = [sum(wr[i, c_] * x[t, c_] for c_ in range(d)) for i in range(E)]
        n = math.sqrt(sum(v * v for v in z))
        s = [sigma * c * max(0.0, v / (n + eps)) for v in z]
        chosen = set(sorted(range(E), key=lambda i: (-z[i], i))[:k])
        out = [0.0] * d
        for i in range(E):                      # every expert, densely; mask by selection
            y = _dense_expert(x[t], wg[i], wu[i], wd[i])
            m = 1.0 if i in chosen else 0.0
            for c_ in range(d):
                out[c_] += m * s[i] * y[c_]
        np.testing.assert_allclose(fw["out"][t], out, rtol=1e-11, atol=1e-13)


def test_single_expert_is_a_dense_swiglu_mlp():
    torch = pytest.importorskip("torch")
    x, wr, wg, wu, wd = tiny(T=9, d=8, f=5, E=1, k=1)
    fw = O.moe_layer_fwd(x, wr, wg, wu, wd, 1, 1.0, 1.0, 0.0)
    xt = torch.tensor(x, dtype=torch.float64)
    mlp = torch.nn.functional.silu(xt @ torch.tensor(wg[0]).T) * (xt @ torch.tensor(wu[0]).T)
    mlp = (mlp @ torch.tensor(wd[0]).T).numpy()
    # with E = 1 and eps = 0 the score is relu(sign(z)): 1 for positive logits, else 0
    gate = (x @ wr[0] > 0).astype(np.float64)[:, None]
    np.testing.assert_allclose(fw["out"], gate * mlp, rtol=1e-12, atol=1e-14)


def test_expert_relabelling_and_token_permutation():
    x, wr, wg, wu, wd = tiny(T=30, d=8, f=6, E=7, k=3)
    args = (3, 1.1, 2.0, 1e-6)
    fw = O.moe_layer_fwd(x, wr, wg, wu, wd, *args)
    rng = np.random.default_rng(5)
    pe = rng.permutation(7)
    fw2 = O.moe_layer_fwd(x, wr[pe], wg[pe], wu[pe], wd[pe], *args)
    np.testing.assert_allclose(fw2["out"], fw["out"], rtol=1e-12, atol=1e-14)
    assert np.array_equal(fw2["counts"], fw["counts"][pe])
    pt = rng.permutation(30)
    fw3 = O.moe_layer_fwd(x[pt], wr, wg, wu, wd, *args)
    np.testing.assert_allclose(fw3["out"], fw["out"][pt], rtol=1e-12, atol=1e-14)
    assert np.array_equal(fw3["counts"], fw["counts"])
    np.testing.assert_allclose(fw3["psum"], fw["psum"], rtol=1e-12)


# ------------------------------------------------------------------ Eq. 4-6
def test_pool_loss_hand_values():
    g = json.load(open(os.path.join(GOLDEN, "normrouter_hand_example.json")))["pool_loss"]
    pc, fbar, loss, coef = O.pool_aux_loss(np.array(g["counts"]), np.array(g["psum"]),
                                           g["T"], g["k"], g["alpha"])
    assert pc.tolist() == g["pool_counts"]
    np.testing.assert_allclose(fbar, g["fbar"], atol=1e-15)
    assert loss == pytest.approx(g["loss"], abs=1e-15)
    np.testing.assert_allclose(coef, g["coef"], atol=1e-15)


def test_pool_loss_closed_forms():
    rng = np.random.default_rng(2)
    L, M, T, k, alpha = 4, 12, 60, 2, 0.02
    psum = rng.random((L, M)) * T
    # (i) exactly uniform pool usage (layers individually skewed): loss = alpha * sum_i Pbar_i
    counts = np.zeros((L, M))
    for l in range(L):
        hot = np.arange(M) % L == l
        counts[l, hot] = T * k / hot.sum()
    assert np.all(counts.sum(axis=0) == counts.sum(axis=0)[0])
    _, fbar, loss, _ = O.pool_aux_loss(counts, psum, T, k, alpha)
    np.testing.assert_allclose(fbar, 1.0 / M, rtol=1e-14)
    assert loss == pytest.approx(alpha * psum.sum() / (L * T), rel=1e-13)
    # rows of scores summing to one -> loss == alpha exactly
    p1 = rng.random((L, T, M))
    p1 /= p1.sum(axis=2, keepdims=True)
    _, _, loss1, _ = O.pool_aux_loss(counts, p1.sum(axis=1), T, k, alpha)
    assert loss1 == pytest.approx(alpha, rel=1e-13)
    # (ii) all traffic on one expert j: loss = alpha * M * Pbar_j
    c2 = np.zeros((L, M))
    c2[:, 5] = T * k
    _, _, loss2, _ = O.pool_aux_loss(c2, psum, T, k, alpha)
    assert loss2 == pytest.approx(alpha * M * psum[:, 5].sum() / (L * T), rel=1e-13)
    # (iii) Eq. 6 == Eq. 5
    c3 = rng.multinomial(T * k, np.ones(M) / M, size=L)
    _, _, loss3, _ = O.pool_aux_loss(c3, psum, T, k, alpha)
    loss3d, per_layer = O.pool_aux_loss_decomposed(c3, psum, T, k, alpha)
    assert loss3 == pytest.approx(loss3d, rel=1e-13) and len(per_layer) == L
    # (iv) L = 1 is the per-layer Switch loss, Eq. 3: alpha * E * sum f_i P_i
    _, _, loss4, _ = O.pool_aux_loss(c3[:1], psum[:1], T, k, alpha)
    f = c3[0] / (T * k)
    P = psum[0] / T
    assert loss4 == pytest.approx(alpha * M * float(f @ P), rel=1e-13)
    # lagged fbar is used as given
    fl = rng.random(M)
    _, fnow, loss5, coef5 = O.pool_aux_loss(c3, psum, T, k, alpha, fbar_in=fl)
    assert loss5 == pytest.approx(alpha * M * float(fl @ (psum / T).mean(axis=0)), rel=1e-13)
    np.testing.assert_allclose(fnow, c3.sum(axis=0) / (L * T * k), rtol=1e-14)
    np.testing.assert_allclose(coef5, alpha * M * fl / (L * T), rtol=1e-14)


def test_counts_sum_and_pool_totals():
    w = W.WORKLOADS["C1"]
    wg, wu, wd = W.gen_pool_weights(w)
    counts = []
    for l in range(w.L):
        fw = O.moe_layer_fwd(W.gen_x(w, l), W.gen_w_router(w, l), wg, wu, wd, w.k, w.sigma, w.c, w.eps)
        assert int(fw["counts"].sum()) == w.T * w.k
        counts.append(fw["counts"])
    pc, fbar, _, _ = O.pool_aux_loss(np.stack(counts), np.zeros((w.L, w.E)), w.T, w.k, w.alpha)
    assert int(pc.sum()) == w.L * w.T * w.k
    assert float(fbar.sum()) == pytest.approx(1.0, abs=1e-14)


# ------------------------------------------------------------------ App. H (NormRouter Monte Carlo initialization)
def test_estimate_c_calibrates_selected_scores():
    # definition of c: mean over tokens of 1/||gate/(sigma c)||_2 on Gaussian logits ~ c
    E, k = 64, 2
    c, used = O.estimate_c(E, k, 100_000, seed=1)
    assert used == 100_000 and 2.60 < c < 2.70
    rng = np.random.default_rng(9)
    z = rng.standard_normal((100_000, E))
    s, _ = O.norm_router_scores(z, 1.0, 1.0, 0.0)
    idx = O.topk_select(z, k)
    g = np.take_along_axis(s, idx.astype(np.int64), axis=1)
    assert np.mean(1.0 / np.linalg.norm(g, axis=1)) == pytest.approx(c, rel=5e-3)
    # E = k = 1: y = relu(sign x) -> 1 for x > 0, dropped otherwise -> c = 1
    c1, used1 = O.estimate_c(1, 1, 2000, seed=0)
    assert c1 == pytest.approx(1.0, abs=1e-15) and 900 < used1 < 1100
