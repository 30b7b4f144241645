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


TOL = {"f32": 1e-5, "bf16": 1e-2}
