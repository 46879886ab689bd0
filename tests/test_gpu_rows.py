"""svgd_step_rows: particles as n separately allocated vectors (App. B.2: the leader gathers every
particle's own flat parameter and gradient vectors) against the oracle and against svgd_step on
the packed matrix."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import svgd_oracle as orc
from parity_checks import TOL_H, TOL_K, assert_x_new, ulp_diff

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svgd():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2306_06528_amd import svgd as mod
    return mod


def _separate_rows(M, seed, aligned=False):
    """Each row of M copied into an allocation of its own, at a different offset from the
    allocation's start (so every row has its own alignment; aligned: offsets of whole 128-byte
    lines, so every row starts on a line boundary), in shuffled allocation order."""
    n, D = M.shape
    rng = np.random.default_rng(seed)
    bufs, rows = [], [None] * n
    for i in rng.permutation(n):
        off = 32 * int(rng.integers(0, 2)) if aligned else int(rng.integers(0, 37))
        b = torch.full((D + 64,), float("nan"), device=M.device)
        assert b.data_ptr() % 128 == 0
        b[off:off + D] = M[i]
        bufs.append(b)
        rows[i] = b[off:off + D]
    return bufs, rows


@pytest.mark.parametrize("n,D", [(1, 1000), (2, 65), (3, 50_003), (8, 70_001), (12, 8577), (13, 4099), (16, 8577),
                                 (17, 20_011), (32, 20_001), (33, 5003), (48, 129), (64, 70_001), (64, 63), (5, 300)])
@pytest.mark.parametrize("aligned", [False, True])
def test_separate_rows_match_oracle_and_packed_step(svgd, n, D, aligned):
    g = torch.Generator(device="cuda")
    g.manual_seed(100 * n + D)
    X0 = torch.randn(n, D, generator=g, device="cuda") * 0.3
    G0 = torch.randn(n, D, generator=g, device="cuda")
    eps = 0.05
    xb, xr = _separate_rows(X0, 1, aligned)
    gb, gr = _separate_rows(G0, 2, aligned)
    Xp = X0.clone()
    with svgd.Svgd(n, D) as eng:
        eng.step_rows(xr, gr, eps)
        h, K = eng.get_last(n)
        eng.step(Xp, G0, eps)
        torch.cuda.synchronize()
    ref = orc.step(X0.cpu().numpy(), G0.cpu().numpy(), eps)
    assert abs(h - ref["h"]) / ref["h"] <= TOL_H
    assert np.abs(K - ref["K"]).max() <= TOL_K
    got = torch.stack(xr).cpu().numpy()
    assert_x_new(got, ref, eps, f"rows n={n} D={D}")
    # the packed step runs the same arithmetic (on another kernel instance, or in the single-launch
    # kernel with its own summation order at the smallest sizes): one rounding of x, or a millionth
    # of eps * max|phi|
    slack = float(np.spacing(np.float32(np.abs(got).max()))) + 1e-6 * eps * float(np.abs(ref["phi"]).max())
    assert np.abs(Xp.cpu().numpy().astype(np.float64) - got).max() <= slack, "separate rows differ from the packed step"
    # nothing outside the rows was written, G untouched
    for b, r in zip(xb, [xr[i] for i in np.random.default_rng(1).permutation(n)]):
        off = r.storage_offset()
        assert torch.isnan(b[:off]).all() and torch.isnan(b[off + D:]).all()
    assert torch.equal(torch.stack(gr), G0)


@pytest.mark.parametrize("aligned", [False, True])
@pytest.mark.parametrize("n,D", [(32, 4_400_003), (17, 5_000_003)])
def test_large_separate_rows(svgd, n, D, aligned):
    """X beyond twice (n = 32) or 1.25 times (n = 17) the memory-side cache as separate rows: the
    sizes at which the pairwise pass reorders and streams its loads and the update shares ranges or
    runs two workgroups per CU.  Against the oracle (h, K, X_new)."""
    g = torch.Generator(device="cuda")
    g.manual_seed(n + D)
    X0 = torch.randn(n, D, generator=g, device="cuda") * 0.05
    G0 = torch.randn(n, D, generator=g, device="cuda") * 1e-2
    eps = 1e-3
    _, xr = _separate_rows(X0, 3, aligned)
    _, gr = _separate_rows(G0, 4, aligned)
    with svgd.Svgd(n, D) as eng:
        eng.step_rows(xr, gr, eps)
        h, K = eng.get_last(n)
        torch.cuda.synchronize()
    ref = orc.step(X0.cpu().numpy(), G0.cpu().numpy(), eps)
    assert abs(h - ref["h"]) / ref["h"] <= TOL_H
    assert np.abs(K - ref["K"]).max() <= TOL_K
    assert_x_new(torch.stack(xr).cpu().numpy(), ref, eps, f"rows n={n} D={D}")


def test_rows_of_one_matrix_are_separate_rows_too(svgd):
    """Rows that happen to be the rows of one matrix: the same call, the same result."""
    n, D = 20, 3001
    X0 = torch.randn(n, D, device="cuda")
    G0 = torch.randn(n, D, device="cuda")
    Xa, Xb = X0.clone(), X0.clone()
    with svgd.Svgd(n, D) as eng:
        eng.step_rows([Xa[i] for i in range(n)], [G0[i] for i in range(n)], 0.01)
        eng.step(Xb, G0, 0.01)
        torch.cuda.synchronize()
    assert ulp_diff(Xb.cpu().numpy().astype(np.float64), Xa.cpu().numpy()) <= 1.0


def test_rows_argument_errors(svgd):
    lib = svgd._lib
    n, D = 4, 100
    X = torch.randn(n, D, device="cuda")
    G = torch.randn(n, D, device="cuda")
    eng = svgd.Svgd(n, D)
    P = ctypes.c_void_p * n
    xp = P(*[X[i].data_ptr() for i in range(n)])
    gp = P(*[G[i].data_ptr() for i in range(n)])
    assert lib.svgd_step_rows(eng._h, None, gp, n, D, 0.1, None) == -1
    assert lib.svgd_step_rows(eng._h, xp, gp, 0, D, 0.1, None) == -1
    assert lib.svgd_step_rows(eng._h, xp, gp, n, D, float("nan"), None) == -1
    assert lib.svgd_step_rows(eng._h, xp, gp, n + 1, D, 0.1, None) == -3
    bad = P(X[0].data_ptr(), 0, X[2].data_ptr(), X[3].data_ptr())             # null row
    assert lib.svgd_step_rows(eng._h, bad, gp, n, D, 0.1, None) == -1
    bad = P(X[0].data_ptr(), X[1].data_ptr() + 2, X[2].data_ptr(), X[3].data_ptr())   # misaligned row
    assert lib.svgd_step_rows(eng._h, bad, gp, n, D, 0.1, None) == -1
    bad = P(X[0].data_ptr(), X[0].data_ptr() + 40, X[2].data_ptr(), X[3].data_ptr())  # rows overlap
    assert lib.svgd_step_rows(eng._h, bad, gp, n, D, 0.1, None) == -1
    assert lib.svgd_step_rows(eng._h, xp, xp, n, D, 0.1, None) == -1                  # G rows are the X rows
    torch.cuda.synchronize()
    assert lib.svgd_step_rows(eng._h, xp, gp, n, D, 0.1, None) == 0
    torch.cuda.synchronize()
    assert torch.isfinite(X).all()
    eng.close()
