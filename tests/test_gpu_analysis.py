"""GPU parity of the analysis observables: Alg. 1 on given draws (App. H (NormRouter Monte Carlo initialization)) and the distinct-expert
count U(x) (App. E (distinct-expert accounting)), through the C ABI, against the oracle."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from synth import workloads as W
from tests.gpu_util import dev, host
from tests.test_gpu_parity import lib, shape_of, workspace

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("E,k,n", [(8, 2, 1000), (5, 1, 77), (192, 2, 100000), (512, 8, 5000), (96, 1, 4097),
                                   (3, 3, 64), (1, 1, 50)])
def test_estimate_c(E, k, n):
    import torch
    U = lib()
    rng = np.random.default_rng(1000 + E + k)
    x = rng.standard_normal((n, E)).astype(np.float32)
    if n > 10:
        x[3] = -np.abs(x[3])                     # a draw with no positive component
    gx = torch.from_numpy(x).cuda()
    c = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    used = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    ws = torch.empty(2 * 256 * ((4 * ((n + 63) // 64) + 255) // 256) + 256, dtype=torch.uint8, device="cuda")
    U.estimate_c(E, k, gx, c, used, ws)
    U.estimate_c(E, k, gx, c, used, ws)           # repeatable
    torch.cuda.synchronize()
    ref_c, ref_used = O.c_from_samples(x, k)
    assert int(used.item()) == ref_used
    assert abs(float(c.item()) - ref_c) <= 1e-5 * ref_c


def test_estimate_c_reproduces_the_workload_constant():
    """The constants of the synthetic workloads were estimated the same way (2e5 draws)."""
    import torch
    U = lib()
    w = W.WORKLOADS["C5"]
    n = 200000
    g = torch.Generator(device="cuda")
    g.manual_seed(5)
    gx = torch.randn((n, w.E), generator=g, device="cuda", dtype=torch.float32)
    c = torch.zeros(1, dtype=torch.float32, device="cuda")
    used = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")
    U.estimate_c(w.E, w.k, gx, c, used, ws)
    torch.cuda.synchronize()
    assert int(used.item()) == n
    assert abs(float(c.item()) - w.c) < 0.01 * w.c


def test_estimate_c_rejects_a_small_workspace():
    import torch
    U = lib()
    gx = torch.zeros((100000, 8), dtype=torch.float32, device="cuda")
    c = torch.zeros(1, dtype=torch.float32, device="cuda")
    used = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(U.UniPoolError):
        U.estimate_c(8, 2, gx, c, used, torch.empty(256, dtype=torch.uint8, device="cuda"))


@pytest.mark.parametrize("T,k,E,L", [(1000, 2, 8, 3), (77, 3, 5, 2), (5000, 1, 192, 24), (300, 8, 512, 4), (1, 1, 1, 1)])
def test_distinct_experts(T, k, E, L):
    import torch
    U = lib()
    rng = np.random.default_rng(T + k + E + L)
    idx = [np.stack([rng.choice(E, size=k, replace=False) for _ in range(T)]).astype(np.int32) for _ in range(L)]
    if L > 1 and T > 1:
        idx[1][0] = idx[0][0]                    # a token that repeats its selection
    gidx = [torch.from_numpy(i).cuda() for i in idx]
    tab = torch.tensor([t.data_ptr() for t in gidx], dtype=torch.int64, device="cuda")
    w = W.Workload("x", L=L, E=E, d=64, f=64, k=k, T=T, dtype="bf16", seed=0)
    sh = shape_of(w)
    dist = torch.full((T,), -1, dtype=torch.int32, device="cuda")
    mean = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    U.distinct_experts(sh, L, tab, dist, mean, workspace(sh))
    torch.cuda.synchronize()
    ref_u, ref_mean = O.distinct_experts(idx)
    assert np.array_equal(host(dist), ref_u)
    assert abs(float(mean.item()) - ref_mean) <= 1e-6 * ref_mean
