"""GPU parity of the one-kernel router (Sec. 4.3, Eq. 7 and the top-k paragraph; softmax scores of the
comparison rows in Sec. 5.4) over every compiled body: the number of 16-expert blocks (pools of 8 to 512
experts, some not multiples of 16), one and two token fragments per wavefront (two need at least 128 tokens
per compute unit of the device, so those cases hold 32768 tokens and a ragged tail), and both prefetch depths
(d_model a multiple of 256 or only of 128).  Logits, scores and statistics against the float64 oracle;
selection bit-exact outside near-ties, a valid choice on them."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import TOL, check_selection, dev, host, rel_err

pytestmark = pytest.mark.gpu

BIG_T = 32768 + 77       # 257 tiles of 128 tokens: at least one per compute unit, the last one ragged
CASES = [
    # (E, k, d_model, T)
    (8, 2, 128, BIG_T), (24, 3, 256, BIG_T), (56, 2, 128, BIG_T), (96, 2, 256, BIG_T), (120, 4, 128, BIG_T),
    (136, 2, 128, BIG_T), (200, 2, 256, BIG_T), (256, 8, 128, BIG_T),
    (8, 1, 256, 130), (40, 2, 128, 333), (64, 2, 384, 1000), (88, 3, 128, 64), (128, 2, 256, 700),
    (192, 2, 128, 129), (248, 5, 256, 500), (264, 2, 128, 400), (384, 8, 256, 777), (392, 3, 128, 65),
    (512, 8, 256, 1111), (512, 2, 128, 63),
]


@pytest.mark.parametrize("router", ["norm", "softmax"])
@pytest.mark.parametrize("E,k,d,T", CASES, ids=["E%d-k%d-d%d-T%d" % c for c in CASES])
def test_fused_router_body(E, k, d, T, router):
    import torch
    import paper_2605_06665_amd as U
    if router == "softmax" and T == BIG_T and E not in (56, 200):
        pytest.skip("the softmax branch shares the kernel bodies: two of the large cases suffice")
    w = W.Workload("router-body", L=1, E=E, d=d, f=64, k=k, T=T, dtype="bf16", seed=1000 + E + k + d, c=2.4)
    sh = U.Shape(T=T, d_model=d, d_ff=64, E=E, k=k, L=1, dtype=U.BF16, sigma=0.9, c=w.c, eps=w.eps,
                 alpha_pool=w.alpha, router=U.ROUTER_SOFTMAX if router == "softmax" else U.ROUTER_NORM)
    assert U.fast_path(sh) & 4, "this shape must take the one-kernel router"
    x, wr = W.gen_x(w, 0), W.gen_w_router(w, 0)
    ref = O.route(x, wr, k, 0.9, w.c, w.eps, router=router)
    xd, wd = dev(x, "bf16"), dev(wr, "bf16")
    idx = torch.full((T, k), -1, dtype=torch.int32, device="cuda")
    gate = torch.full((T, k), float("nan"), device="cuda")
    logits = torch.full((T, E), float("nan"), device="cuda")
    counts = torch.full((E,), -1, dtype=torch.int32, device="cuda")
    psum = torch.full((E,), float("nan"), device="cuda")
    ws = torch.empty(U.workspace_bytes(sh), dtype=torch.uint8, device="cuda")
    U.route(sh, xd, wd, idx, gate, logits, counts, psum, ws)
    torch.cuda.synchronize()
    tol = TOL["bf16"]
    assert rel_err(host(logits), ref["z"]) <= tol
    gi = host(idx)
    # outside near-ties bit-exact, on them a valid choice; gates = the oracle's scores of the chosen experts
    # (both score functions keep the order of the logits, so one selection rule serves both)
    check_selection(ref["z"], ref["idx"], gi, k, scores=ref["s"], got_gate=host(gate), tol=tol)
    assert np.array_equal(host(counts), np.bincount(gi.ravel(), minlength=E))
    assert int(host(counts).sum()) == T * k
    assert rel_err(host(psum), ref["psum"]) <= tol
