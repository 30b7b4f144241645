"""Helpers of the GPU parity tests: numpy <-> device tensors and the error metric."""
import numpy as np


def has_gpu():
    try:
        import torch
        return torch.cuda.is_available()
    except Exception:
        return False


def dev(a, dtype=None):
    """numpy array -> cuda tensor.  dtype "bf16" converts exactly-representable float32 values."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    elif dtype == "f32":
        t = t.to(torch.float32)
    return t.contiguous()


def host(t):
    import torch
    if t.dtype == torch.bfloat16:
        t = t.to(torch.float32)
    return t.detach().cpu().numpy()


def round_act(a, dtype):
    """float64 oracle values -> float32 values representable in the activation dtype."""
    from synth import workloads as W
    return W.round_to_dtype(np.asarray(a, dtype=np.float32), dtype)


def rel_err(got, ref):
    """max |got - ref| / max |ref| per tensor (the tolerance of the parity bar is on this)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    scale = float(np.max(np.abs(ref)))
    if scale == 0.0:
        return float(np.max(np.abs(got)))
    return float(np.max(np.abs(got - ref))) / scale


def near_tie_tokens(z64, k, sigma_unused=None, tol=1e-6):
    """Tokens whose top-(k+1) normalised logits hold an adjacent pair closer than tol."""
    z64 = np.asarray(z64, dtype=np.float64)
    n = np.sqrt(np.sum(z64 * z64, axis=1, keepdims=True))
    zh = z64 / np.where(n > 0, n, 1.0)
    srt = -np.sort(-zh, axis=1)
    top = srt[:, :min(k + 1, zh.shape[1])]
    return np.min(-np.diff(top, axis=1), axis=1) < tol if top.shape[1] > 1 else np.zeros(len(zh), bool)


def check_selection(z64, ref_idx, got_idx, k, scores=None, got_gate=None, tol=1e-5, tie_tol=1e-6):
    """Compares a selection with the oracle's and returns (tie mask, index array to hand on).

    Outside near-tie tokens the indices must equal the oracle's bit for bit.  On a near-tie token
    several answers are correct, so the check says which: k distinct experts in range, every chosen
    expert's float64 normalised logit at least the oracle's k-th largest minus tie_tol, slots in
    descending order (to tie_tol), and - when scores [T, E] (the oracle's) and got_gate are given -
    the gate of every slot equal to the oracle's score of the expert chosen there.  The returned
    indices are the oracle's with the checked choice taken over on the near-tie tokens only."""
    z64 = np.asarray(z64, dtype=np.float64)
    ref_idx, got_idx = np.asarray(ref_idx), np.asarray(got_idx)
    T, E = z64.shape
    tie = near_tie_tokens(z64, k, tol=tie_tol)
    assert np.array_equal(got_idx[~tie], ref_idx[~tie]), "top-k indices differ outside near-ties"
    merged = ref_idx.copy()
    if tie.any():
        n = np.sqrt(np.sum(z64 * z64, axis=1, keepdims=True))
        zh = (z64 / np.where(n > 0, n, 1.0))[tie]
        gi = got_idx[tie]
        assert gi.min() >= 0 and gi.max() < E, "near-tie token with an expert out of range"
        assert all(len(set(r)) == k for r in gi.tolist()), "near-tie token with a repeated expert"
        kth = -np.sort(-zh, axis=1)[:, k - 1]
        chosen = np.take_along_axis(zh, gi, axis=1)
        assert (chosen >= kth[:, None] - tie_tol).all(), "near-tie token holds an expert below the k-th largest logit"
        assert (np.diff(chosen, axis=1) <= tie_tol).all(), "near-tie token: slots not in descending order"
        merged[tie] = gi
    if scores is not None and got_gate is not None:
        want = np.take_along_axis(np.asarray(scores, dtype=np.float64), merged.astype(np.int64), axis=1)
        assert rel_err(got_gate, want) <= tol, "gates differ from the oracle's scores of the chosen experts"
    return tie, merged


TOL = {"f32": 1e-5, "bf16": 1e-2}
