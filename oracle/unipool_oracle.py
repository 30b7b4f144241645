"""CPU oracle for the shared-pool MoE layer (UniPool) -- TEST INFRASTRUCTURE ONLY.

A plain, slow, float64 statement of what the layer computes, written from the
paper's equations.  It shares no code with the GPU path and must never be used
by it: only the tests, the smoke check and the benchmark's CPU-baseline leg call
into this module.

Every function states the passage it follows.  numpy's matmul, sort and cumsum
serve as steps; there is no blocking, fusion or reordering beyond the equations.

Readings taken where the paper leaves a choice (all are inputs or one-liners):
  * selection is on the logits z (monotone in the score s for sigma*c > 0),
    exact ties go to the lower expert index, slots are in descending order;
  * gates are the raw scores s of the selected experts (no renormalisation);
  * epsilon is added outside the norm, as printed in Eq. 7;
  * f_i^(l) = (slots of layer l routed to i) / (T k), so that sum_i f_i = 1;
  * P_i^(l) = (1/T) sum_t s_{t,i} over all experts, unmasked;
  * SwiGLU expert: e(x) = W_down ( silu(W_gate x) * (W_up x) ), no bias;
  * inside an expert's group rows are ordered by ascending token index.

Weights use the Linear convention [out_features, in_features].

Pins (tests/test_oracle_*.py): dense brute force of Eq. 2 with Python loops,
full-sort top-k, permutation invariants, NormRouter closed forms, pool-loss
closed forms (uniform usage, single expert, L = 1 reducing to Eq. 3, Eq. 6
identity), central finite differences for every gradient, E = 1 reducing to a
dense SwiGLU MLP; the softmax router (comparison rows of Sec. 5.4) by rows summing to one, the
pool loss equal to alpha under exactly uniform usage, shift invariance and finite differences;
the one-step-behind loop against a hand count of the previous
micro-batch's slots and finite differences of the lagged objective; the
recompute half against the forward record.  `c_from_samples` (App. H (NormRouter Monte Carlo initialization), Alg. 1) is pinned by
loops on small draws and closed cases, `estimate_c` statistically; `distinct_experts`
(App. E (distinct-expert accounting)) by hand cases and the occupancy closed form for uniform routing.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# ---------------------------------------------------------------------------
# Router (Sec. 4.3, Eq. 7) and top-k selection
# ---------------------------------------------------------------------------
def router_logits(x, w_router):
    """z = W h for every token (Sec. 4.3): x [T,d], w_router [E,d] -> [T,E]."""
    return np.asarray(x, F64) @ np.asarray(w_router, F64).T


def norm_router_scores(z, sigma, c, eps):
    """Eq. 7: s_i = sigma * c * max(0, z_i / (||z||_2 + eps)).  Returns (s, ||z||)."""
    z = np.asarray(z, F64)
    n = np.sqrt(np.sum(z * z, axis=-1))
    zhat = z / (n + eps)[..., None]
    return sigma * c * np.maximum(0.0, zhat), n


def softmax_router_scores(z):
    """The softmax router of the comparison rows (Sec. 4.1, Eq. 1 and Sec. 4.2, Eq. 3; Sec. 5.4 ablation
    "softmax router"): p_i = exp(z_i) / sum_j exp(z_j).  The gate of a selected expert is
    its probability p_i (no renormalisation over the top-k: with the paper's top-1 routing a
    renormalised gate would be the constant 1 and the router would get no gradient from
    the layer output), and the auxiliary losses use p as the routing probability."""
    z = np.asarray(z, F64)
    e = np.exp(z - np.max(z, axis=-1, keepdims=True))
    return e / np.sum(e, axis=-1, keepdims=True)


def router_scores(z, sigma, c, eps, router="norm"):
    """Scores of the router kind: "norm" is Eq. 7, "softmax" the softmax router."""
    if router == "norm":
        return norm_router_scores(z, sigma, c, eps)
    assert router == "softmax", router
    z = np.asarray(z, F64)
    return softmax_router_scores(z), np.sqrt(np.sum(z * z, axis=-1))


def topk_select(z, k):
    """Indices of the k largest logits per token, descending, ties -> lower index."""
    z = np.asarray(z, F64)
    order = np.argsort(-z, axis=-1, kind="stable")
    return order[..., :k].astype(np.int32)


def route(x, w_router, k, sigma, c, eps, idx=None, router="norm"):
    """Router of one layer: logits, scores, top-k, gates and the layer statistics
    the auxiliary losses need (Sec. 4.2: token counts per expert and the sum of
    routing scores per expert over the tokens of the layer).
    `idx` replaces the selection (used by tests to impose the other, equally
    valid choice on tokens whose logits tie within rounding)."""
    z = router_logits(x, w_router)
    s, n = router_scores(z, sigma, c, eps, router)
    idx = topk_select(z, k) if idx is None else np.asarray(idx, dtype=np.int32)
    gate = np.take_along_axis(s, idx.astype(np.int64), axis=1)
    E = z.shape[1]
    counts = np.bincount(idx.ravel(), minlength=E).astype(np.int64)
    psum = s.sum(axis=0)
    return dict(z=z, norm=n, s=s, idx=idx, gate=gate, counts=counts, psum=psum)


# ---------------------------------------------------------------------------
# Dispatch: expert-contiguous permutation
# ---------------------------------------------------------------------------
def permutation(idx, E):
    """Row layout of the expert-contiguous token copy.

    offsets[e] .. offsets[e+1] are the rows of expert e; inside a group rows
    are in ascending token order.  slot = t*k + j.
    Returns (offsets[E+1], row_of_slot[T,k], slot_of_row[T*k])."""
    idx = np.asarray(idx)
    T, k = idx.shape
    counts = np.bincount(idx.ravel(), minlength=E)
    offsets = np.zeros(E + 1, dtype=np.int64)
    offsets[1:] = np.cumsum(counts)
    slot_of_row = np.empty(T * k, dtype=np.int64)
    fill = offsets[:-1].copy()
    for t in range(T):                 # ascending token order inside each group
        for j in range(k):
            e = idx[t, j]
            slot_of_row[fill[e]] = t * k + j
            fill[e] += 1
    row_of_slot = np.empty(T * k, dtype=np.int64)
    row_of_slot[slot_of_row] = np.arange(T * k)
    return offsets, row_of_slot.reshape(T, k), slot_of_row


def permute_rows(x, slot_of_row, k):
    """x_perm[row] = x[token of that row]."""
    return np.asarray(x)[np.asarray(slot_of_row) // k]


# ---------------------------------------------------------------------------
# SwiGLU experts (Table 6 caption: SwiGLU FFN) and the layer output (Eq. 2)
# ---------------------------------------------------------------------------
def logistic(a):
    a = np.asarray(a, F64)
    return 1.0 / (1.0 + np.exp(-a))


def silu(a):
    return np.asarray(a, F64) * logistic(a)


def silu_grad(a):
    sg = logistic(a)
    return sg * (1.0 + np.asarray(a, F64) * (1.0 - sg))


def expert_apply(x_rows, w_gate_e, w_up_e, w_down_e):
    """One expert on a block of rows.  Returns (a, b, h, y)."""
    x_rows = np.asarray(x_rows, F64)
    a = x_rows @ np.asarray(w_gate_e, F64).T
    b = x_rows @ np.asarray(w_up_e, F64).T
    h = silu(a) * b
    y = h @ np.asarray(w_down_e, F64).T
    return a, b, h, y


def expert_ffn_fwd(x_perm, offsets, w_gate, w_up, w_down):
    """Every pool expert on its own group of rows."""
    S = x_perm.shape[0]
    E, f, d = w_gate.shape
    a = np.zeros((S, f), F64)
    b = np.zeros((S, f), F64)
    h = np.zeros((S, f), F64)
    y = np.zeros((S, d), F64)
    for e in range(E):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 > r0:
            a[r0:r1], b[r0:r1], h[r0:r1], y[r0:r1] = expert_apply(
                x_perm[r0:r1], w_gate[e], w_up[e], w_down[e])
    return a, b, h, y


def expert_ffn_recompute(x_perm, offsets, w_gate, w_up):
    """App. C (activation checkpointing with MoE recompute): A, B and H of every group
    again from the kept rows -- the gate and up projections and the SwiGLU product of
    expert_ffn_fwd, without the down projection."""
    x_perm = np.asarray(x_perm, F64)
    S = x_perm.shape[0]
    E, f, _ = w_gate.shape
    a = np.zeros((S, f), F64)
    b = np.zeros((S, f), F64)
    for e in range(E):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 > r0:
            a[r0:r1] = x_perm[r0:r1] @ np.asarray(w_gate[e], F64).T
            b[r0:r1] = x_perm[r0:r1] @ np.asarray(w_up[e], F64).T
    return a, b, silu(a) * b


def combine(y_perm, row_of_slot, gate=None):
    """Eq. 2: out_t = sum_j g_{t,j} * y_perm[row(t,j)]  (gate None = unit gates)."""
    y_perm = np.asarray(y_perm, F64)
    T, k = row_of_slot.shape
    out = np.zeros((T, y_perm.shape[1]), F64)
    for j in range(k):
        rows = y_perm[row_of_slot[:, j]]
        out += rows if gate is None else np.asarray(gate, F64)[:, j:j + 1] * rows
    return out


def moe_layer_fwd(x, w_router, w_gate, w_up, w_down, k, sigma, c, eps, idx=None, router="norm"):
    """Eq. 2 for one layer, through routing, dispatch, experts and combine."""
    E = w_gate.shape[0]
    r = route(x, w_router, k, sigma, c, eps, idx, router)
    offsets, row_of_slot, slot_of_row = permutation(r["idx"], E)
    x_perm = permute_rows(np.asarray(x, F64), slot_of_row, k)
    a, b, h, y = expert_ffn_fwd(x_perm, offsets, w_gate, w_up, w_down)
    out = combine(y, row_of_slot, r["gate"])
    r.update(offsets=offsets, row_of_slot=row_of_slot, slot_of_row=slot_of_row,
             x_perm=x_perm, a=a, b=b, h=h, y_perm=y, out=out)
    return r


# ---------------------------------------------------------------------------
# Pool-level auxiliary loss (Sec. 4.2, Eq. 4-6; App. G (pool auxiliary loss derivation))
# ---------------------------------------------------------------------------
def pool_aux_loss(counts, psum, T, k, alpha, fbar_in=None):
    """counts [L,E] slot counts, psum [L,E] score sums.

    f_i^(l) = counts/(T k);  fbar = mean_l f^(l)   (Eq. 4), unless a lagged
    fbar is supplied (App. G (pool auxiliary loss derivation), one-step-behind: fbar is a constant either way);
    P_i^(l) = psum/T;  Pbar = mean_l P^(l);
    loss = alpha * M * sum_i fbar_i * Pbar_i        (Eq. 5).
    coef_i = d loss / d s_{t,i}^(l) = alpha * M * fbar_i / (L T)   (from Eq. 6).
    Returns (pool_counts[E], fbar_same_step[E], loss, coef[E])."""
    counts = np.asarray(counts, F64)
    psum = np.asarray(psum, F64)
    L, M = counts.shape
    f = counts / float(T * k)
    fbar_now = f.mean(axis=0)
    fbar = fbar_now if fbar_in is None else np.asarray(fbar_in, F64)
    pbar = (psum / float(T)).mean(axis=0)
    loss = alpha * M * float(np.sum(fbar * pbar))
    coef = alpha * M * fbar / float(L * T)
    return counts.sum(axis=0).astype(np.int64), fbar_now, loss, coef


def pool_aux_loss_decomposed(counts, psum, T, k, alpha, fbar_in=None):
    """Eq. 6: the same loss as the mean over layers of per-layer contributions."""
    counts = np.asarray(counts, F64)
    psum = np.asarray(psum, F64)
    L, M = counts.shape
    fbar = (counts / float(T * k)).mean(axis=0) if fbar_in is None else np.asarray(fbar_in, F64)
    per_layer = [alpha * M * float(np.sum(fbar * (psum[l] / float(T)))) for l in range(L)]
    return sum(per_layer) / L, per_layer


# ---------------------------------------------------------------------------
# Backward (derivatives of Eq. 2, Eq. 7 and Eq. 6; App. G (pool auxiliary loss derivation): only the routing
# scores carry the auxiliary gradient)
# ---------------------------------------------------------------------------
def combine_bwd(dout, y_perm, row_of_slot, gate):
    """d y_perm[row(t,j)] = g_{t,j} dout_t ;  d g_{t,j} = <dout_t, y_perm[row(t,j)]>."""
    dout = np.asarray(dout, F64)
    y_perm = np.asarray(y_perm, F64)
    gate = np.asarray(gate, F64)
    T, k = row_of_slot.shape
    dy = np.zeros_like(y_perm)
    dgate = np.zeros((T, k), F64)
    for j in range(k):
        rows = row_of_slot[:, j]
        dy[rows] = gate[:, j:j + 1] * dout
        dgate[:, j] = np.sum(dout * y_perm[rows], axis=1)
    return dy, dgate


def expert_ffn_bwd(dy_perm, x_perm, a, b, offsets, w_gate, w_up, w_down):
    """Gradients of y = W_down (silu(W_gate x) * (W_up x)) per expert group.
    Returns (dx_perm, dw_gate, dw_up, dw_down, da, db)."""
    dy_perm = np.asarray(dy_perm, F64)
    x_perm = np.asarray(x_perm, F64)
    a = np.asarray(a, F64)
    b = np.asarray(b, F64)
    E = w_gate.shape[0]
    dx = np.zeros_like(x_perm)
    da = np.zeros_like(a)
    db = np.zeros_like(b)
    dwg = np.zeros(w_gate.shape, F64)
    dwu = np.zeros(w_up.shape, F64)
    dwd = np.zeros(w_down.shape, F64)
    for e in range(E):
        r0, r1 = int(offsets[e]), int(offsets[e + 1])
        if r1 == r0:
            continue
        xe, ae, be, dye = x_perm[r0:r1], a[r0:r1], b[r0:r1], dy_perm[r0:r1]
        he = silu(ae) * be
        dh = dye @ np.asarray(w_down[e], F64)            # [r, f]
        dwd[e] = dye.T @ he                              # [d, f]
        dae = dh * be * silu_grad(ae)
        dbe = dh * silu(ae)
        dwg[e] = dae.T @ xe                              # [f, d]
        dwu[e] = dbe.T @ xe
        dx[r0:r1] = dae @ np.asarray(w_gate[e], F64) + dbe @ np.asarray(w_up[e], F64)
        da[r0:r1], db[r0:r1] = dae, dbe
    return dx, dwg, dwu, dwd, da, db


def route_bwd(x, w_router, z, idx, dgate, aux_coef, sigma, c, eps, router="norm"):
    """Backward of Eq. 7 (or of the softmax router) and of z = W h.

    ds_{t,i} = aux_coef_i (every expert; zero if aux_coef is None)
               + dgate_{t,j} where i = idx_{t,j};
    d sigma = sum ds * c * relu(zhat);  dzhat = ds * sigma c [zhat > 0];
    dz_j = dzhat_j/(n+eps) - z_j <dzhat, z> / (n (n+eps)^2);
    dW = dz^T x;  dx = dz W.
    router = "softmax":  dz_j = p_j (ds_j - <ds, p>)  (Jacobian of the softmax), d sigma = 0.
    Returns (dx[T,d], dw_router[E,d], dsigma, dz[T,E])."""
    x = np.asarray(x, F64)
    w_router = np.asarray(w_router, F64)
    z = np.asarray(z, F64)
    T, E = z.shape
    ds = np.zeros((T, E), F64)
    if aux_coef is not None:
        ds += np.asarray(aux_coef, F64)[None, :]
    dgate = np.asarray(dgate, F64)
    for j in range(idx.shape[1]):
        ds[np.arange(T), idx[:, j]] += dgate[:, j]
    if router == "softmax":
        p = softmax_router_scores(z)
        dz = p * (ds - np.sum(ds * p, axis=1, keepdims=True))
        return dz @ w_router, dz.T @ x, 0.0, dz
    assert router == "norm", router
    n = np.sqrt(np.sum(z * z, axis=1))
    zhat = z / (n + eps)[:, None]
    pos = zhat > 0.0
    dsigma = float(np.sum(ds * c * np.maximum(0.0, zhat)))
    dzhat = np.where(pos, ds * sigma * c, 0.0)
    dot = np.sum(dzhat * z, axis=1)
    safe_n = np.where(n > 0.0, n, 1.0)
    dz = dzhat / (n + eps)[:, None] - z * (dot / (safe_n * (n + eps) ** 2))[:, None]
    dz[n == 0.0] = 0.0
    dw = dz.T @ x
    dx = dz @ w_router
    return dx, dw, dsigma, dz


def moe_layer_bwd(fw, x, w_router, w_gate, w_up, w_down, dout, aux_coef, k, sigma, c, eps, router="norm"):
    """Backward of one layer given its forward record `fw` (from moe_layer_fwd)."""
    dy, dgate = combine_bwd(dout, fw["y_perm"], fw["row_of_slot"], fw["gate"])
    dxp, dwg, dwu, dwd, da, db = expert_ffn_bwd(dy, fw["x_perm"], fw["a"], fw["b"], fw["offsets"],
                                                w_gate, w_up, w_down)
    dx_experts = combine(dxp, fw["row_of_slot"], None)       # sum over the k copies
    dx_router, dwr, dsigma, dz = route_bwd(x, w_router, fw["z"], fw["idx"], dgate, aux_coef,
                                           sigma, c, eps, router)
    return dict(dy_perm=dy, dgate=dgate, dx_perm=dxp, da=da, db=db, dw_gate=dwg, dw_up=dwu,
                dw_down=dwd, dx_experts=dx_experts, dx_router=dx_router,
                dx=dx_experts + dx_router, dw_router=dwr, dsigma=dsigma, dz=dz)


# ---------------------------------------------------------------------------
# Whole step over the L layers that share the pool
# ---------------------------------------------------------------------------
def pool_step(xs, w_routers, w_gate, w_up, w_down, grad_outs, k, sigmas, c, eps, alpha,
              fbar_in=None, idxs=None, aux="pool", router="norm"):
    """Forward of all layers, auxiliary loss, backward of all layers.
    Expert weight gradients are summed over the layers (one shared pool).

    aux = "pool":  the pool-level loss of Eq. 5 over all the layers;
    aux = "layer": the per-layer loss of Eq. 3 for every layer on its own, each entering the
                   objective with weight one (the ablation row "shared pool + layer aux",
                   Sec. 5.4); "loss" is then their sum, "loss_layers" the list, and "coef"
                   holds one coefficient vector per layer."""
    L = len(xs)
    T = xs[0].shape[0]
    fws = [moe_layer_fwd(xs[l], w_routers[l], w_gate, w_up, w_down, k, sigmas[l], c, eps,
                         None if idxs is None else idxs[l], router)
           for l in range(L)]
    counts = np.stack([fw["counts"] for fw in fws])
    psum = np.stack([fw["psum"] for fw in fws])
    loss_layers = None
    if aux == "pool":
        pool_counts, fbar, loss, coef = pool_aux_loss(counts, psum, T, k, alpha, fbar_in)
        coefs = [coef] * L
    else:
        assert aux == "layer" and fbar_in is None
        per = [pool_aux_loss(counts[l:l + 1], psum[l:l + 1], T, k, alpha) for l in range(L)]
        pool_counts = counts.sum(axis=0).astype(np.int64)
        fbar = np.stack([p[1] for p in per])                 # f^(l), one row per layer
        loss_layers = [p[2] for p in per]
        loss = float(sum(loss_layers))
        coefs = [p[3] for p in per]
        coef = np.stack(coefs)
    dwg = np.zeros(w_gate.shape, F64)
    dwu = np.zeros(w_up.shape, F64)
    dwd = np.zeros(w_down.shape, F64)
    bws = []
    for l in range(L):
        bw = moe_layer_bwd(fws[l], xs[l], w_routers[l], w_gate, w_up, w_down, grad_outs[l], coefs[l],
                           k, sigmas[l], c, eps, router)
        dwg += bw["dw_gate"]
        dwu += bw["dw_up"]
        dwd += bw["dw_down"]
        bws.append(bw)
    return dict(fw=fws, bw=bws, counts=counts, psum=psum, pool_counts=pool_counts, fbar=fbar,
                loss=loss, loss_layers=loss_layers, coef=coef, dw_gate=dwg, dw_up=dwu, dw_down=dwd)


def pool_groups_step(groups, k, c, eps, alpha, router="norm"):
    """Sharing scope G (Sec. 5.4): the layers are cut into G groups over depth, every group
    routes into a pool of its own and carries its own pool loss (Eq. 5 over the group's
    layers); G = 1 is the fully shared pool, one layer per group is the layer-private MoE
    with the loss of Eq. 3 (with router = "softmax" and k = 1 that is the vanilla MoE of Eq. 1
    that the paper compares against).  `groups` is a list of dicts with keys xs, w_routers,
    w_gate, w_up, w_down, grad_outs, sigmas.  Returns the per-group pool_step results and the
    sum of the group losses."""
    results = [pool_step(g["xs"], g["w_routers"], g["w_gate"], g["w_up"], g["w_down"], g["grad_outs"],
                         k, g["sigmas"], c, eps, alpha, router=router) for g in groups]
    return results, float(sum(r["loss"] for r in results))


def micro_batch_loop(batches, w_routers, w_gate, w_up, w_down, k, sigmas, c, eps, alpha, fbar0=None):
    """App. G (pool auxiliary loss derivation), one-step-behind: micro-batch m takes the usage statistic fbar of micro-batch
    m-1 as a constant; the first one takes `fbar0`, or, when that is None, its own (the
    paper does not say what the first micro-batch uses).  `batches` is a list of
    (xs, grad_outs).  Returns the list of pool_step results; entry m's "fbar" is the
    statistic that micro-batch m+1 uses."""
    results = []
    fbar = fbar0
    for xs, grad_outs in batches:
        r = pool_step(xs, w_routers, w_gate, w_up, w_down, grad_outs, k, sigmas, c, eps, alpha,
                      fbar_in=fbar)
        results.append(r)
        fbar = r["fbar"]
    return results


def objective(xs, w_routers, w_gate, w_up, w_down, grad_outs, k, sigmas, c, eps, alpha, fbar, router="norm"):
    """Lambda = sum_l <Out^(l), G^(l)> + L_pool with fbar held constant (App. G (pool auxiliary loss derivation))."""
    total = 0.0
    psum = []
    for l in range(len(xs)):
        fw = moe_layer_fwd(xs[l], w_routers[l], w_gate, w_up, w_down, k, sigmas[l], c, eps, None, router)
        total += float(np.sum(fw["out"] * np.asarray(grad_outs[l], F64)))
        psum.append(fw["psum"])
    psum = np.stack(psum)
    T = xs[0].shape[0]
    M = w_gate.shape[0]
    pbar = (psum / float(T)).mean(axis=0)
    return total + alpha * M * float(np.sum(np.asarray(fbar, F64) * pbar))


# ---------------------------------------------------------------------------
# App. H (NormRouter Monte Carlo initialization), Alg. 1: Monte-Carlo estimate of the NormRouter constant c
# ---------------------------------------------------------------------------
def c_from_samples(samples, k):
    """App. H (NormRouter Monte Carlo initialization), Alg. 1 on given draws x ~ N(0, I_E), one per row: for every row
    y = relu(x / ||x||_2), the k largest components of y, 1 / their 2-norm; c is the mean.
    Rows whose top-k part is all zero (1/0) are dropped; the paper does not treat that
    case.  Returns (c, rows_used)."""
    x = np.asarray(samples, F64)
    y = np.maximum(0.0, x / np.linalg.norm(x, axis=1, keepdims=True))
    ysort = -np.sort(-y, axis=1)
    nrm = np.sqrt(np.sum(ysort[:, :k] ** 2, axis=1))
    ok = nrm > 0.0
    return float(np.mean(1.0 / nrm[ok])), int(ok.sum())


def estimate_c(E, k, n_samples=100_000, seed=0):
    """Alg. 1 with its own draws.  Returns (c, samples_used)."""
    rng = np.random.default_rng(seed)
    return c_from_samples(rng.standard_normal((n_samples, E)), k)


# ---------------------------------------------------------------------------
# App. E (distinct-expert accounting): distinct experts touched by a token over the layers that share a pool
# ---------------------------------------------------------------------------
def distinct_experts(idx_layers):
    """U(x) = | { experts selected for token x at any of the L layers } |  (App. E (distinct-expert accounting); stated
    there for top-1, taken here over all k selections of every layer).
    idx_layers: L arrays [T, k].  Returns (U [T] int64, mean of U)."""
    idx = np.stack([np.asarray(i) for i in idx_layers], axis=1)      # [T, L, k]
    T = idx.shape[0]
    U = np.array([len(set(idx[t].ravel().tolist())) for t in range(T)], dtype=np.int64)
    return U, float(U.mean())
