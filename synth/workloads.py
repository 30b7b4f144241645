"""Seeded synthetic workloads for the shared-pool MoE layer.

This module is the only code shared by the CPU oracle's tests and the GPU path's
tests/bench.  It holds shapes, seeds, value distributions and dtype conversion
(float32 <-> bfloat16 bit patterns) and nothing of the method itself: no router,
no top-k, no expert arithmetic.

Shapes follow the five benchmark configurations (C1..C5).  The paper trains on
the Pile with Megatron-LM (Sec. 5.1, Tables 7-8); those token streams and trained
weights are not available, so every tensor here is drawn from a stated
distribution with a stated seed and stands in for them.

Tensor conventions (all row-major):
  x[l]        [T, d]     token hidden states entering layer l        N(0, 1)
  w_router[l] [E, d]     router matrix W of layer l (Sec. 4.3)       N(0, 1)
  grad_out[l] [T, d]     upstream gradient of the layer output       N(0, 1)
  w_gate      [E, f, d]  SwiGLU gate projection, Linear convention   N(0, 0.02^2)
  w_up        [E, f, d]  SwiGLU up projection                        N(0, 0.02^2)
  w_down      [E, d, f]  SwiGLU down projection                      N(0, 0.02^2)
"Linear convention" = [out_features, in_features]:  a = x @ w_gate[e].T.

Expert-preference skew (stand-in for the uneven per-layer usage the paper shows
in Fig. 4): the last input feature is set to the constant 1 and the last column
of w_router[l] carries a per-expert offset  sqrt(d-1) * bias_i, so that
logit_i / sqrt(d-1) = bias_i + N(0,1) noise.  The offsets are fixed constants,
calibrated offline with plain Gaussian sampling:
  "hot":  a per-layer random 20 % of the experts get bias 0.625, which makes
          them take ~50 % of the top-2 slots at E = 96;
  "zipf": bias_i = 0.5 * log p_i with p_i ~ rank_i^-1.1 over a per-layer random
          ranking (tail experts end with a handful of rows).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

# tensor ids used in seed derivation
_ID_X, _ID_WR, _ID_WG, _ID_WU, _ID_WD, _ID_G, _ID_SKEW = range(7)


@dataclass(frozen=True)
class Workload:
    name: str
    L: int          # layers sharing the pool
    E: int          # pool size M
    d: int          # d_model
    f: int          # d_ff of one expert
    k: int          # top-k
    T: int          # tokens per layer call
    dtype: str      # "f32" or "bf16"
    seed: int
    sigma: float = 1.0       # NormRouter learnable scale at init (Sec. 4.3)
    c: float = 1.0           # NormRouter calibration constant (App. H (NormRouter Monte Carlo initialization)), an input here
    eps: float = 1e-6        # NormRouter epsilon
    alpha: float = 1e-2      # pool auxiliary loss coefficient (Table 8)
    skew: str = "none"       # "none" | "hot" | "hot_shared" | "zipf"

    @property
    def S(self) -> int:
        return self.T * self.k

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


# c(E, k): Monte-Carlo estimates of App. H (NormRouter Monte Carlo initialization)'s expectation (2e5 samples); they are
# plain inputs to both the oracle and the GPU path.
WORKLOADS: Dict[str, Workload] = {
    "C1": Workload("C1-tiny-f32", L=2, E=8, d=64, f=128, k=2, T=128, dtype="f32",
                   seed=0, c=2.5, alpha=1e-2),
    "C2": Workload("C2-small-bf16", L=8, E=64, d=768, f=2048, k=2, T=8192,
                   dtype="bf16", seed=1, c=2.652, alpha=1e-2),
    "C3": Workload("C3-reduced-pool-bf16", L=16, E=96, d=1024, f=2816, k=2,
                   T=16384, dtype="bf16", seed=2, c=3.022, alpha=2e-2, skew="hot"),
    "C3s": Workload("C3-reduced-pool-shared-hot-bf16", L=16, E=96, d=1024, f=2816,
                    k=2, T=16384, dtype="bf16", seed=2, c=3.022, alpha=2e-2,
                    skew="hot_shared"),
    "C4": Workload("C4-fine-grained-uniform-bf16", L=16, E=512, d=1024, f=704, k=8,
                   T=16384, dtype="bf16", seed=3, c=3.204, alpha=2e-2),
    "C4z": Workload("C4-fine-grained-zipf-bf16", L=16, E=512, d=1024, f=704, k=8,
                    T=16384, dtype="bf16", seed=3, c=3.204, alpha=2e-2, skew="zipf"),
    "C5": Workload("C5-largest-bf16", L=24, E=192, d=1536, f=4096, k=2, T=32768,
                   dtype="bf16", seed=4, c=3.847, alpha=2e-2),
}

HOT_FRACTION = 0.2
HOT_BIAS = 0.625
ZIPF_EXPONENT = 1.1
ZIPF_GAMMA = 0.5
WEIGHT_STD = 0.02


# --------------------------------------------------------------------------
# bfloat16 bit conversion (format conversion only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), returned as uint16."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    out = ((u + rounding) >> 16).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        out[nan] = 0x7FC0
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    """Return float32 values representable in `dtype` ("f32" leaves them as is)."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(a))
    return a


# --------------------------------------------------------------------------
# numpy backend (host; used up to C2-sized tensors and by all CPU tests)
# --------------------------------------------------------------------------
def _rng(w: Workload, tensor_id: int, layer: int = 0) -> np.random.Generator:
    return np.random.default_rng([w.seed, tensor_id, layer])


def expert_bias(w: Workload, layer: int) -> Optional[np.ndarray]:
    """Per-expert logit offsets (in units of the noise std) of layer `layer`."""
    if w.skew == "none":
        return None
    lay = 0 if w.skew == "hot_shared" else layer
    rng = _rng(w, _ID_SKEW, lay)
    perm = rng.permutation(w.E)
    bias = np.zeros(w.E, dtype=np.float64)
    if w.skew in ("hot", "hot_shared"):
        n_hot = max(1, int(round(HOT_FRACTION * w.E)))
        bias[perm[:n_hot]] = HOT_BIAS
    elif w.skew == "zipf":
        p = np.arange(1, w.E + 1, dtype=np.float64) ** (-ZIPF_EXPONENT)
        p /= p.sum()
        bias[perm] = ZIPF_GAMMA * np.log(p)
    else:
        raise ValueError(w.skew)
    return bias


def gen_x(w: Workload, layer: int) -> np.ndarray:
    x = _rng(w, _ID_X, layer).standard_normal((w.T, w.d), dtype=np.float32)
    if w.skew != "none":
        x[:, w.d - 1] = 1.0
    return round_to_dtype(x, w.dtype)


def gen_w_router(w: Workload, layer: int) -> np.ndarray:
    wr = _rng(w, _ID_WR, layer).standard_normal((w.E, w.d), dtype=np.float32)
    bias = expert_bias(w, layer)
    if bias is not None:
        wr[:, w.d - 1] = (math.sqrt(w.d - 1) * bias).astype(np.float32)
    return round_to_dtype(wr, w.dtype)


def gen_grad_out(w: Workload, layer: int) -> np.ndarray:
    g = _rng(w, _ID_G, layer).standard_normal((w.T, w.d), dtype=np.float32)
    return round_to_dtype(g, w.dtype)


def gen_pool_weights(w: Workload):
    """(w_gate[E,f,d], w_up[E,f,d], w_down[E,d,f]) float32, representable in w.dtype."""
    wg = _rng(w, _ID_WG).standard_normal((w.E, w.f, w.d), dtype=np.float32) * np.float32(WEIGHT_STD)
    wu = _rng(w, _ID_WU).standard_normal((w.E, w.f, w.d), dtype=np.float32) * np.float32(WEIGHT_STD)
    wd = _rng(w, _ID_WD).standard_normal((w.E, w.d, w.f), dtype=np.float32) * np.float32(WEIGHT_STD)
    return round_to_dtype(wg, w.dtype), round_to_dtype(wu, w.dtype), round_to_dtype(wd, w.dtype)


# --------------------------------------------------------------------------
# torch backend (tensors drawn on the device; for workloads too large to draw
# on the host).  The oracle side receives host copies of the slices it needs.
# --------------------------------------------------------------------------
def _torch_dtype(w: Workload):
    import torch
    return torch.bfloat16 if w.dtype == "bf16" else torch.float32


def _torch_normal(w: Workload, shape, tensor_id: int, layer: int, device, std: float = 1.0):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(w.seed * 100003 + tensor_id * 1009 + layer)
    out = torch.empty(shape, dtype=torch.float32, device=device)
    out.normal_(0.0, std, generator=g)
    return out


def gen_x_torch(w: Workload, layer: int, device):
    x = _torch_normal(w, (w.T, w.d), _ID_X, layer, device)
    if w.skew != "none":
        x[:, w.d - 1] = 1.0
    return x.to(_torch_dtype(w))


def gen_w_router_torch(w: Workload, layer: int, device):
    import torch
    wr = _torch_normal(w, (w.E, w.d), _ID_WR, layer, device)
    bias = expert_bias(w, layer)
    if bias is not None:
        wr[:, w.d - 1] = torch.from_numpy((math.sqrt(w.d - 1) * bias).astype(np.float32)).to(device)
    return wr.to(_torch_dtype(w))


def gen_grad_out_torch(w: Workload, layer: int, device):
    return _torch_normal(w, (w.T, w.d), _ID_G, layer, device).to(_torch_dtype(w))


def gen_pool_weights_torch(w: Workload, device):
    """Drawn expert by expert to bound the float32 staging memory."""
    import torch
    dt = _torch_dtype(w)
    wg = torch.empty((w.E, w.f, w.d), dtype=dt, device=device)
    wu = torch.empty((w.E, w.f, w.d), dtype=dt, device=device)
    wd = torch.empty((w.E, w.d, w.f), dtype=dt, device=device)
    for e in range(w.E):
        wg[e] = _torch_normal(w, (w.f, w.d), _ID_WG, e, device, WEIGHT_STD).to(dt)
        wu[e] = _torch_normal(w, (w.f, w.d), _ID_WU, e, device, WEIGHT_STD).to(dt)
        wd[e] = _torch_normal(w, (w.d, w.f), _ID_WD, e, device, WEIGHT_STD).to(dt)
    return wg, wu, wd
