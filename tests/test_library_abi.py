"""Host-side checks of the C-ABI library: it loads, exports every function the header declares,
and rejects bad shapes without touching a GPU."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def U():
    import __graft_entry__ as g
    g.ensure_built()
    import paper_2605_06665_amd as U
    U.load_library()
    return U


def declared_functions():
    text = open(os.path.join(ROOT, "include", "unipool.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(unipool_[a-z_0-9]+)\s*\(", text)))


def test_header_functions_are_exported(U):
    names = declared_functions()
    assert len(names) >= 12
    lib = U.load_library()
    for n in names:
        assert hasattr(lib, n), n
    from paper_2605_06665_amd import binding
    assert sorted(binding.ENTRY_POINTS) == names


def test_workspace_size_and_shape_validation(U):
    sh = U.Shape(T=128, d_model=64, d_ff=128, E=8, k=2, L=2, dtype=U.F32, sigma=1.0, c=2.5, eps=1e-6,
                 alpha_pool=0.01)
    n = U.workspace_bytes(sh)
    assert n > 0 and n % 256 == 0
    big = U.Shape(T=32768, d_model=1536, d_ff=4096, E=192, k=2, L=24, dtype=U.BF16, sigma=1.0, c=3.8,
                  eps=1e-6, alpha_pool=0.02)
    assert U.workspace_bytes(big) > n
    for field, value, msg in (("k", 9, "k=9"), ("E", 513, "E=513"), ("T", 0, "positive"),
                              ("dtype", 7, "dtype"), ("sigma", -1.0, "sigma")):
        bad = U.Shape(T=128, d_model=64, d_ff=128, E=8, k=2, L=2, dtype=U.F32, sigma=1.0, c=2.5, eps=1e-6,
                      alpha_pool=0.01)
        setattr(bad, field, value)
        with pytest.raises(U.UniPoolError, match=msg):
            U.workspace_bytes(bad)
    bad = U.Shape(T=128, d_model=100, d_ff=128, E=8, k=2, L=2, dtype=U.BF16, sigma=1.0, c=2.5, eps=1e-6,
                  alpha_pool=0.01)
    with pytest.raises(U.UniPoolError, match="multiples of 64"):
        U.workspace_bytes(bad)


def test_null_arguments_fail_before_any_launch(U):
    sh = U.Shape(T=128, d_model=64, d_ff=128, E=8, k=2, L=2, dtype=U.F32, sigma=1.0, c=2.5, eps=1e-6,
                 alpha_pool=0.01)
    with pytest.raises(U.UniPoolError, match="NULL"):
        U.combine(sh, None, None, None, None, stream=0)
    with pytest.raises(U.UniPoolError, match="NULL"):
        U.pool_aux_loss(sh, None, None, None, None, None, None, None, stream=0)
    assert "NULL" in U.last_error()


def test_fast_path_reports_the_kernel_families(U):
    def sh(**kw):
        base = dict(T=512, d_model=128, d_ff=192, E=64, k=2, L=2, dtype=U.BF16, sigma=1.0, c=2.5, eps=1e-6,
                    alpha_pool=0.01)
        base.update(kw)
        return U.Shape(**base)
    assert U.fast_path(sh()) == 7                       # MFMA experts, MFMA router, fused router
    assert U.fast_path(sh(E=512)) == 7                  # the largest pool the fused router takes
    assert U.fast_path(sh(d_model=192)) == 3            # d_model not a multiple of 128: logits GEMM and selection in two kernels
    assert U.fast_path(sh(E=10)) == 1                   # E not a multiple of 8: plain router kernels
    assert U.fast_path(sh(dtype=U.F32)) == 0            # float mode: plain kernels throughout
    with pytest.raises(U.UniPoolError, match="k=9"):
        U.fast_path(sh(k=9))
