"""unipool_permute_static (the entry point that allocates nothing: its scratch is a static device
array inside the library) against unipool_permute, through the C ABI: bit-exact integer outputs and
row copies, two calls in a row on the same GPU, the second with a smaller input, so that whatever
the first call left in the shared scratch must not reach the second call's results."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import dev, host

pytestmark = pytest.mark.gpu

BIG = W.Workload("static-big", L=1, E=48, d=128, f=64, k=3, T=4200, dtype="bf16", seed=31, c=2.5, skew="hot")
SMALL = W.Workload("static-small", L=1, E=48, d=128, f=64, k=3, T=333, dtype="bf16", seed=32, c=2.5)


def _run_pair(w):
    import torch
    import paper_2605_06665_amd as U
    sh = U.Shape(T=w.T, d_model=w.d, d_ff=w.f, E=w.E, k=w.k, L=w.L, dtype=U.BF16, sigma=w.sigma, c=w.c,
                 eps=w.eps, alpha_pool=w.alpha)
    x_h = W.gen_x(w, 0)
    r = O.route(x_h, W.gen_w_router(w, 0), w.k, w.sigma, w.c, w.eps)
    x = dev(x_h, "bf16")
    idx, cnt = dev(r["idx"].astype(np.int32)), dev(r["counts"].astype(np.int32))

    def outputs():
        return (torch.full((w.S, w.d), float("nan"), dtype=torch.bfloat16, device="cuda"),
                torch.full((w.E + 1,), -1, dtype=torch.int32, device="cuda"),
                torch.full((w.T, w.k), -1, dtype=torch.int32, device="cuda"),
                torch.full((w.S,), -1, dtype=torch.int32, device="cuda"))
    ref = outputs()
    ws = torch.empty(U.workspace_bytes(sh), dtype=torch.uint8, device="cuda")
    U.permute(sh, x, idx, cnt, *ref, ws)
    got = outputs()
    U.permute_static(sh, x, idx, cnt, *got)
    torch.cuda.synchronize()
    for a, b, name in zip(got, ref, ("x_perm", "expert_offsets", "row_of_slot", "slot_of_row")):
        assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                           b.view(torch.int16) if b.dtype == torch.bfloat16 else b), (w.name, name)
    # and both against the oracle's permutation
    off, ros, sor = O.permutation(r["idx"], w.E)
    assert np.array_equal(host(got[1]), off) and np.array_equal(host(got[2]), ros)
    assert np.array_equal(host(got[3]), sor)
    assert np.array_equal(host(got[0]), O.permute_rows(x_h, sor, w.k))


def test_permute_static_matches_permute_twice_in_a_row():
    _run_pair(BIG)
    _run_pair(SMALL)      # smaller input right after: the scratch still holds the first call's histograms


def test_permute_static_rejects_shapes_beyond_its_scratch():
    import torch
    import paper_2605_06665_amd as U
    sh = U.Shape(T=1 << 17, d_model=64, d_ff=64, E=512, k=1, L=1, dtype=U.BF16, sigma=1.0, c=2.0, eps=1e-6,
                 alpha_pool=0.01)        # ceil(T/64) * E = 2^20 words > 2^19
    x = torch.empty(8, dtype=torch.int32, device="cuda")
    with pytest.raises(U.UniPoolError, match="exceeds the static scratch"):
        U.permute_static(sh, x, x, x, x, x, x, x)
