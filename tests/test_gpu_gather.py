"""GPU parity of the fused dispatch of the forward pass: unipool_permute without a permuted copy (index maps
only) and unipool_expert_ffn_fwd_gather, whose first GEMM reads the rows of x through slot_of_row.  Results
must be bitwise those of the path with the materialised copy, and meet the oracle at the usual bar."""
import numpy as np
import pytest

from oracle import unipool_oracle as O
from tests.gpu_util import TOL, dev, host, rel_err
from tests.test_gpu_parity import _ffn_inputs, empty, lib, oracle_case, pack_gate_up, shape_of, workspace

pytestmark = pytest.mark.gpu

NAMES = ["C1", "f32-ragged", "bf16-tiles", "bf16-skew", "bf16-empty", "bf16-k8", "bf16-longk", "bf16-kE", "bf16-T1"]


@pytest.mark.parametrize("name", NAMES)
def test_forward_with_gathered_dispatch(name):
    import torch
    c = oracle_case(name)
    w, U = c["w"], lib()
    sh = shape_of(w)
    r, off, ros, sor, x_perm = _ffn_inputs(c)
    a, b, h, y = O.expert_ffn_fwd(x_perm, off, c["wg"], c["wu"], c["wd"])
    ws = workspace(sh)
    x = dev(c["xs"][0], w.dtype)
    g_off, g_ros, g_sor = empty((w.E + 1,), "i32"), empty((w.T, w.k), "i32"), empty((w.S,), "i32")
    U.permute(sh, None, dev(r["idx"].astype(np.int32)), dev(r["counts"].astype(np.int32)), None, g_off, g_ros, g_sor,
              ws)                                       # index maps only
    torch.cuda.synchronize()
    assert np.array_equal(host(g_off), off) and np.array_equal(host(g_ros), ros) and np.array_equal(host(g_sor), sor)
    wgu, wd = dev(pack_gate_up(c["wg"], c["wu"]), w.dtype), dev(c["wd"], w.dtype)
    outs = []
    for gather in (False, True):
        ga, gb, gh = (empty((w.S, w.f), w.dtype) for _ in range(3))
        gy = empty((w.S, w.d), w.dtype)
        for t in (ga, gb, gh, gy):
            t.fill_(float("nan"))
        if gather:
            U.expert_ffn_fwd_gather(sh, x, g_sor, g_off, wgu, wd, ga, gb, gh, gy, ws)
        else:
            U.expert_ffn_fwd(sh, dev(x_perm, w.dtype), g_off, wgu, wd, ga, gb, gh, gy, ws)
        torch.cuda.synchronize()
        outs.append((ga, gb, gh, gy))
    tol = TOL[w.dtype]
    for got, mat, ref, nm in zip(outs[1], outs[0], (a, b, h, y), "abhy"):
        assert torch.equal(got.view(torch.int16) if got.dtype == torch.bfloat16 else got,
                           mat.view(torch.int16) if mat.dtype == torch.bfloat16 else mat), nm
        assert np.isfinite(host(got)).all() and rel_err(host(got), ref) <= tol, nm
