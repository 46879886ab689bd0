"""svgd_step_static, the entry point that allocates nothing (static device scratch inside the
library), against svgd_step_ld on a handle: same kernels, so the same X, through the C ABI.
Two calls in a row on the same GPU, the second with a smaller input, so that whatever the first
call left in the shared scratch is there when the second one runs."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import svgd_oracle as orc
from parity_checks import assert_x_new, ulp_diff

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svgd():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2306_06528_amd import svgd as mod
    return mod


def _problem(n, D, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn(n, D, generator=g, device="cuda") * 0.3, torch.randn(n, D, generator=g, device="cuda")


def _one(svgd, n, D, seed, eps=0.05):
    lib = svgd._lib
    X0, G = _problem(n, D, seed)
    Xs, Xh = X0.clone(), X0.clone()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.svgd_step_static(Xs.data_ptr(), G.data_ptr(), n, D, D, eps, stream)
    assert rc == 0, svgd.status_string(rc)
    with svgd.Svgd(n, D) as eng:
        rc = lib.svgd_step_ld(eng._h, Xh.data_ptr(), G.data_ptr(), n, D, D, eps, stream)
        assert rc == 0
        torch.cuda.synchronize()
    a, b = Xs.cpu().numpy(), Xh.cpu().numpy()
    assert np.isfinite(a).all()
    assert ulp_diff(b.astype(np.float64), a) <= 1.0, "static-scratch step differs from the handle's step"
    # and both against the oracle, at the phi tolerance
    ref = orc.step(X0.cpu().numpy(), G.cpu().numpy(), eps)
    assert_x_new(a, ref, eps, f"static n={n} D={D}")


@pytest.mark.parametrize("first,second", [((64, 70_001), (32, 4099)), ((8, 300_007), (4, 1024)),
                                          ((48, 20_011), (16, 8577)), ((12, 50_003), (64, 63))])
def test_two_calls_in_a_row_second_smaller(svgd, first, second):
    _one(svgd, *first, seed=11)
    _one(svgd, *second, seed=12)


def test_limits_and_errors(svgd):
    lib = svgd._lib
    X, G = _problem(4, 100, 3)
    xp, gp = X.data_ptr(), G.data_ptr()
    assert lib.svgd_step_static(None, gp, 4, 100, 100, 0.1, None) == -1
    assert lib.svgd_step_static(xp, gp, 0, 100, 100, 0.1, None) == -1
    assert lib.svgd_step_static(xp, gp, 4, 100, 99, 0.1, None) == -1          # ld < D
    assert lib.svgd_step_static(xp, xp, 4, 100, 100, 0.1, None) == -1          # X aliases G
    assert lib.svgd_step_static(xp, gp, 4, 100, 100, float("nan"), None) == -1
    assert lib.svgd_step_static(xp, gp, 65, 100, 100, 0.1, None) == -3         # beyond SVGD_MAX_PARTICLES
    assert lib.svgd_step_static(xp, gp, 4, svgd.STATIC_MAX_D + 1, svgd.STATIC_MAX_D + 1, 0.1, None) == -3
    torch.cuda.synchronize()
    assert torch.isfinite(X).all()


def test_static_step_allocates_nothing(svgd):
    """Device memory in use (as the driver reports it) does not change across calls once the first
    call on the device has been made."""
    X, G = _problem(64, 200_003, 5)
    svgd.step_static(X, G, 0.01)
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(5):
        svgd.step_static(X, G, 0.01)
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free1 == free0
