"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle, element by element.

Tolerances (the stated bar): max|dphi| / max|phi| <= 1e-4, |dh| / h <= 1e-5, max|dK| <= 1e-5.
Because eps*phi is only a few ulp of X at NN-like scales, phi is compared through the emit-phi
variant of the same kernels (svgd_phi), and the in-place path (svgd_step) is then checked
against fl32(x + eps * phi_gpu) to one ulp.
"""
import math

import numpy as np
import pytest
import torch

from oracle import svgd_oracle as orc
from paper_2306_06528_amd import workloads
from parity_checks import (TOL_PHI, TOL_H, TOL_K, assert_x_new, check_carried_chain, oracle_kernel_matrix,
                           padded_copy, phi_error_all_columns, ulp_diff as _ulp_diff, ulp_diff_device)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def svgd():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2306_06528_amd import svgd as mod   # raises if libsvgd.so is missing
    return mod


def check_one_step(svgd, X0, G, eps, h_fixed=0.0, tol_phi=TOL_PHI):
    """Runs svgd_phi and svgd_step on (X0, G) and compares with the oracle.  Returns errors."""
    n, D = X0.shape
    Xh, Gh = X0.cpu().numpy(), G.cpu().numpy()
    ref = orc.step(Xh, Gh, eps, h_fixed=h_fixed, want_xnew=False)
    PHI = torch.full_like(X0, float("nan"))
    X = X0.clone()
    with svgd.Svgd(n, D) as eng:
        if h_fixed > 0:
            eng.set_bandwidth(h_fixed)
        h_bw = eng.bandwidth(X)
        eng.phi(X, G, PHI)
        h, K = eng.get_last(n)
        assert torch.equal(X, X0), "svgd_phi must leave X untouched"
        eng.step(X, G, eps)
        torch.cuda.synchronize()
    assert h_bw == h
    phi = PHI.cpu().numpy().astype(np.float64)
    assert np.isfinite(phi).all()
    scale = np.abs(ref["phi"]).max()
    e_phi = np.abs(phi - ref["phi"]).max() / (scale if scale > 0 else 1.0)
    e_l2 = np.linalg.norm(phi - ref["phi"]) / max(np.linalg.norm(ref["phi"]), 1e-300)
    e_h = abs(h - ref["h"]) / ref["h"]
    e_K = np.abs(K.astype(np.float64) - ref["K"]).max()
    assert e_h <= TOL_H, f"h: {h} vs {ref['h']} (rel {e_h:.3e})"
    assert e_K <= TOL_K, f"K: max abs err {e_K:.3e}"
    assert np.array_equal(K, K.T) and np.all(np.diag(K) == 1.0)
    assert e_phi <= tol_phi, f"phi: max err / max|phi| = {e_phi:.3e} (l2 rel {e_l2:.3e})"
    # in-place path: x_new = fl32(fma(eps, phi_gpu, x_old)), allow 1 ulp
    want = Xh.astype(np.float64) + np.float64(np.float32(eps)) * phi
    ulps = _ulp_diff(want, X.cpu().numpy())
    assert ulps <= 1.0, f"in-place update differs from x + eps*phi by {ulps} ulp"
    return dict(e_phi=e_phi, e_l2=e_l2, e_h=e_h, e_K=e_K)


def _random_problem(n, D, seed, x_std=1.0, device="cuda"):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    X = torch.randn(n, D, generator=g, device=device) * x_std
    G = torch.randn(n, D, generator=g, device=device)
    return X, G


# every particle count takes its own template instance / row masking: cover them all at one
# ragged D, and a set of D around the tile sizes (4, 64, 128, 256 columns) at a few n.
# D = 1531 puts n <= 8 on the single-launch path (n * D <= 16384), D = 20011 puts every n on the
# multi-kernel path.
@pytest.mark.parametrize("D", [1531, 20_011])
@pytest.mark.parametrize("n", list(range(1, 18)) + [24, 31, 32, 33, 47, 48, 49, 63, 64])
def test_every_particle_count(svgd, n, D):
    X, G = _random_problem(n, D, 1000 + n + D)
    check_one_step(svgd, X, G, 0.01)


@pytest.mark.parametrize("n,D", [(1, 16_384), (1, 16_385), (2, 8192), (2, 8193), (4, 4096), (4, 4097),
                                 (5, 3276), (5, 3277), (7, 2340), (7, 2341), (8, 2048), (8, 2049),
                                 (8, 1), (3, 2), (6, 7)])
def test_single_launch_path_and_its_size_limit(svgd, n, D):
    """Both sides of n * D = 16384, where the single-workgroup kernel hands over to the
    multi-kernel path, and the smallest shapes."""
    X, G = _random_problem(n, D, 17 * n + D)
    if n > 1 and D < 4:
        X = X * 3.0
    check_one_step(svgd, X, G, 0.05)
    check_one_step(svgd, X, G, 0.05, h_fixed=2.0)


def test_single_launch_and_carried_sums_do_not_mix(svgd):
    """A handle that carries pair sums is used on a large problem, then a tiny one, then the large
    one again: the tiny step must not leave sums behind that the large one would take for its own."""
    nL, DL = 8, 50_021
    XL, GL = _random_problem(nL, DL, 5, x_std=0.3)
    XT, GT = _random_problem(4, 1024, 6, x_std=0.3)
    with svgd.Svgd(8, DL, flags=svgd.FLAG_CARRY_GRAM) as eng:
        eng.step(XL, GL, 0.05)
        for X, G, n in ((XT, GT, 4), (XL, GL, nL), (XT, GT, 4), (XT, GT, 4), (XL, GL, nL), (XL, GL, nL)):
            Xh = X.cpu().numpy()
            eng.step(X, G, 0.05)
            h, K = eng.get_last(n)
            ref = orc.step(Xh, G.cpu().numpy(), 0.05)
            assert abs(h - ref["h"]) / ref["h"] <= TOL_H
            assert np.abs(K - ref["K"]).max() <= TOL_K
            assert_x_new(X.cpu().numpy(), ref, 0.05, f"n={n}")


@pytest.mark.parametrize("n", [1, 2, 4, 8, 13, 16, 20, 32, 40, 64])
@pytest.mark.parametrize("D", [1, 2, 3, 4, 5, 63, 64, 65, 127, 128, 129, 255, 257, 1024, 8577, 70001])
def test_ragged_lengths(svgd, n, D):
    X, G = _random_problem(n, D, 7 * n + D)
    if n > 1 and D < 4:
        # few columns: d2 can be tiny relative to |x|^2; keep the problem well conditioned
        X = X * 3.0
    check_one_step(svgd, X, G, 0.05)


@pytest.mark.parametrize("n", [4, 8, 16, 32, 64])
def test_many_tiles(svgd, n):
    """Several persistent-grid iterations per workgroup and a ragged tail."""
    D = 3_000_017 if n <= 16 else 1_000_003
    X, G = _random_problem(n, D, 99 + n, x_std=0.02)
    G = G * 1e-3
    check_one_step(svgd, X, G, 1e-4)


@pytest.mark.parametrize("n", [3, 8, 16, 32, 64])
def test_translated_particles(svgd, n):
    """A common offset 10x the spread must not spoil d2 (centred / direct-difference Gram)."""
    X, G = _random_problem(n, 4099, 5 + n)
    t = torch.full((1, 4099), 10.0, device="cuda")
    check_one_step(svgd, X + t, G, 0.01, tol_phi=TOL_PHI)


def test_coincident_particles(svgd):
    """All particles equal: med = 0 -> h = 1, K = 1, phi_i = mean_j g_j."""
    x = torch.randn(1, 301, device="cuda")
    for n in (2, 5, 16, 32):
        X = x.repeat(n, 1).contiguous()
        G = torch.randn(n, 301, device="cuda")
        PHI = torch.empty_like(X)
        with svgd.Svgd(n, 301) as eng:
            eng.phi(X, G, PHI)
            h, K = eng.get_last(n)
        assert h == 1.0 and np.all(K == 1.0)
        want = G.double().mean(0, keepdim=True).repeat(n, 1)
        err = (PHI.double() - want).abs().max().item() / want.abs().max().item()
        assert err <= TOL_PHI


@pytest.mark.parametrize("n,groups", [(64, 2), (64, 3), (64, 8), (33, 4), (16, 2), (12, 3), (8, 2), (4, 2)])
def test_clustered_particles_heavy_ties(svgd, n, groups):
    """Groups of identical particles: d2 takes few distinct values, each many times over (and many
    exact zeros), so the two middle order statistics sit inside, or right at the edge of, long runs
    of ties - the median selection has to count them exactly."""
    D = 3001
    centres = torch.randn(groups, D, device="cuda")
    idx = torch.arange(n, device="cuda") % groups
    X = centres[idx].contiguous()
    G = torch.randn(n, D, device="cuda")
    check_one_step(svgd, X, G, 0.01)


@pytest.mark.parametrize("n", [64, 40, 32, 20])
@pytest.mark.parametrize("c", [5.0, 40.0])
def test_outlier_particles_nested_scales(svgd, n, c):
    """A few particles far away from the rest, at two scales: nearly all pairwise distances crowd
    into a sliver of the value range, so the selection has to refine its buckets more than once.
    (Each outlier is displaced along one coordinate of its own by a multiple of n, which shifts
    that column's mean by c or 3c only and keeps the fp32 centred Gram of the other particles
    well conditioned: this is a test of the selection, not of d2.)"""
    D = 2051
    X, G = _random_problem(n, D, 3 * n, x_std=1.0)
    X[0, 0] += c * n
    X[1, 1] += 3 * c * n
    X[2, 2] -= c * n
    check_one_step(svgd, X.contiguous(), G, 0.01)


def test_single_particle_is_gradient_ascent(svgd):
    X, G = _random_problem(1, 1000, 3)
    X0 = X.clone()
    with svgd.Svgd(1, 1000) as eng:
        eng.step(X, G, 0.25)
        h, K = eng.get_last(1)
    assert h == 1.0 and K.tolist() == [[1.0]]
    want = torch.addcmul(X0, G, torch.tensor(0.25, device="cuda"))
    assert _ulp_diff(want.cpu().numpy().astype(np.float64), X.cpu().numpy()) <= 1.0


@pytest.mark.parametrize("n", [4, 16, 32])
def test_fixed_bandwidth(svgd, n):
    """The paper's fixed-lengthscale kernel: h = 2 l^2 given, no median."""
    X, G = _random_problem(n, 2049, 17 + n, x_std=0.1)
    ell = 4.0
    check_one_step(svgd, X, G, 1e-3, h_fixed=2 * ell * ell)


@pytest.mark.parametrize("n,D", [(4, 1000), (8, 50_003), (16, 8577), (64, 20_001)])
def test_fixed_bandwidth_limits(svgd, n, D):
    """h very large: K = 1 and phi_i = mean_j g_j;  h very small: K = I and phi_i = g_i / n (the
    repulsive coefficient (2/h)/n then multiplies x_i - x_i, which the kernels evaluate as a
    difference of two equal products)."""
    X, G = _random_problem(n, D, 41 * n + D)
    PHI = torch.empty_like(X)
    with svgd.Svgd(n, D) as eng:
        eng.set_bandwidth(1e30)
        eng.phi(X, G, PHI)
        h, K = eng.get_last(n)
        assert h == 1e30 and np.all(K == 1.0)
        want = G.double().mean(0, keepdim=True).expand(n, D)
        assert (PHI.double() - want).abs().max().item() / want.abs().max().item() <= TOL_PHI
        eng.set_bandwidth(0.05)          # d2 is about 2 D: exp(-d2 / h) underflows to 0
        eng.phi(X, G, PHI)
        h, K = eng.get_last(n)
        assert h == 0.05 and np.array_equal(K, np.eye(n, dtype=np.float32))
        want = G.double() / n
        assert (PHI.double() - want).abs().max().item() / want.abs().max().item() <= TOL_PHI


def test_handle_reuse_across_shapes(svgd):
    """One handle, several (n, D) in a row: no state leaks from one call to the next."""
    with svgd.Svgd(64, 50_000) as eng:
        for n, D in ((64, 50_000), (3, 17), (32, 4097), (8, 50_000), (17, 129)):
            X, G = _random_problem(n, D, n * D % 1000)
            PHI = torch.empty_like(X)
            eng.phi(X, G, PHI)
            h, K = eng.get_last(n)
            ref = orc.step(X.cpu().numpy(), G.cpu().numpy(), 0.0, want_xnew=False)
            assert abs(h - ref["h"]) / ref["h"] <= TOL_H
            assert np.abs(K - ref["K"]).max() <= TOL_K
            e = np.abs(PHI.cpu().numpy() - ref["phi"]).max() / np.abs(ref["phi"]).max()
            assert e <= TOL_PHI


def test_stream_argument(svgd):
    """Work is enqueued on the stream that is passed in."""
    X, G = _random_problem(8, 100_000, 21)
    X0 = X.clone()
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with svgd.Svgd(8, 100_000) as eng:
        with torch.cuda.stream(s):
            eng.step(X, G, 0.01, stream=s)
        s.synchronize()
    ref = orc.step(X0.cpu().numpy(), G.cpu().numpy(), 0.01)
    assert_x_new(X.cpu().numpy(), ref, 0.01)


# ----------------------------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------------------------
def test_config1_tiny_trajectory(svgd):
    """n=4, D=1024, 200 steps on N(mu, I): teacher-forced parity every step, free-running
    drift at the end, and the particle mean converging to mu."""
    wl = workloads.make(1, device="cuda")
    X = wl.X0.clone()
    Xref = wl.X0.cpu().numpy().astype(np.float64)
    mu = wl.mu.cpu().numpy().astype(np.float64)
    n, D = X.shape
    PHI = torch.empty_like(X)
    err0 = np.linalg.norm(Xref.mean(0) - mu)
    with svgd.Svgd(n, D) as eng:
        for step in range(wl.cfg.steps):
            G = wl.score(X, step)
            eng.phi(X, G, PHI)
            h, K = eng.get_last(n)
            ref = orc.step(X.cpu().numpy(), G.cpu().numpy(), wl.cfg.eps, want_xnew=False)
            assert abs(h - ref["h"]) / ref["h"] <= TOL_H
            assert np.abs(K - ref["K"]).max() <= TOL_K
            e = np.abs(PHI.cpu().numpy() - ref["phi"]).max() / np.abs(ref["phi"]).max()
            assert e <= TOL_PHI, f"step {step}: {e:.3e}"
            eng.step(X, G, wl.cfg.eps)
            Xref = orc.step(Xref, -(Xref - mu), wl.cfg.eps, want_phi=False)["X_new"]
    Xg = X.cpu().numpy().astype(np.float64)
    drift = np.abs(Xg - Xref).max() / np.abs(Xref).max()
    assert drift <= 1e-4, f"free-running drift {drift:.3e}"
    err = np.linalg.norm(Xg.mean(0) - mu)
    assert err / math.sqrt(D) <= 0.05 and err < 0.1 * err0


def test_config2_pinn_mlp_trajectory(svgd):
    """n=16, D=8577 (odd D: rows only 4-byte aligned), 1000 steps; parity checked every 50."""
    wl = workloads.make(2, device="cuda")
    X = wl.X0.clone()
    n, D = X.shape
    PHI = torch.empty_like(X)
    Xref = wl.X0.cpu().numpy().astype(np.float64)
    mu = wl.mu.cpu().numpy().astype(np.float64)
    is2 = wl.inv_sigma2.cpu().numpy().astype(np.float64)
    with svgd.Svgd(n, D) as eng:
        for step in range(wl.cfg.steps):
            G = wl.score(X, step)
            if step % 50 == 0 or step == wl.cfg.steps - 1:
                eng.phi(X, G, PHI)
                h, K = eng.get_last(n)
                ref = orc.step(X.cpu().numpy(), G.cpu().numpy(), wl.cfg.eps, want_xnew=False)
                assert abs(h - ref["h"]) / ref["h"] <= TOL_H
                assert np.abs(K - ref["K"]).max() <= TOL_K
                e = np.abs(PHI.cpu().numpy() - ref["phi"]).max() / np.abs(ref["phi"]).max()
                assert e <= TOL_PHI, f"step {step}: {e:.3e}"
            eng.step(X, G, wl.cfg.eps)
            if step < 100:   # free-running oracle for the first 100 steps
                Xref = orc.step(Xref, (mu - Xref) * is2, wl.cfg.eps, want_phi=False)["X_new"]
                if step == 99:
                    drift = np.abs(X.cpu().numpy() - Xref).max() / np.abs(Xref).max()
                    assert drift <= 1e-4, f"free-running drift after 100 steps {drift:.3e}"


def _plain_step_check(svgd, X0, G, eps, padded=False):
    """One step of a plain handle (the four-kernel step of the four-call ABI) on dense rows or on
    rows padded to 128 bytes: h and K against the oracle's full d2, phi on ALL columns against the
    oracle (streamed in chunks, the normaliser is the oracle's max|phi|), and the in-place update
    == fl32(x + eps * phi_gpu) to one ulp on all n * D entries."""
    n, D = X0.shape
    if padded:
        X, Gv = padded_copy(svgd, X0), padded_copy(svgd, G)
        PHI = svgd.padded_rows(n, D, device=X0.device, fill=float("nan"))
    else:
        X, Gv, PHI = X0.clone(), G, torch.empty_like(X0)
    with svgd.Svgd(n, D) as eng:
        eng.phi(X, Gv, PHI)
        h, K = eng.get_last(n)
        eng.step(X, Gv, eps)
        torch.cuda.synchronize()
    Xh, Gh = X0.cpu().numpy(), G.cpu().numpy()
    h_ref, K_ref = oracle_kernel_matrix(Xh)
    assert abs(h - h_ref) / h_ref <= TOL_H, f"h {h} vs {h_ref}"
    assert np.abs(K - K_ref).max() <= TOL_K
    e_phi = phi_error_all_columns(PHI, Xh, Gh, K_ref, h_ref)
    assert e_phi <= TOL_PHI, f"phi err / max|phi| = {e_phi:.3e}"
    ulps = ulp_diff_device(X, X0, PHI, eps)
    assert ulps <= 1.0, f"in-place update differs from x + eps*phi_gpu by {ulps} ulp"


def _full_size_check(svgd, cfg_index):
    """Full-size config, dense rows, plain handle."""
    wl = workloads.make(cfg_index, device="cuda")
    _plain_step_check(svgd, wl.X0, wl.score(wl.X0, 0), wl.cfg.eps)


def test_config3_operator_net_full_size(svgd):
    _full_size_check(svgd, 3)


def test_config4_resnet18_full_size(svgd):
    _full_size_check(svgd, 4)


def test_config5_large_ensemble_full_size(svgd):
    _full_size_check(svgd, 5)


def _padded(t, ld, sentinel):
    """An (n, D) view with row stride ld of a buffer whose padding holds a sentinel."""
    n, D = t.shape
    buf = torch.full((n, ld), sentinel, device=t.device, dtype=t.dtype)
    buf[:, :D] = t
    return buf, buf[:, :D]


@pytest.mark.parametrize("carry", [False, True])
@pytest.mark.parametrize("n,D,ld", [(4, 1000, 1024), (4, 1000, 1003), (8, 70_001, 70_016), (8, 70_001, 70_002),
                                    (12, 5000, 5024), (16, 8577, 8608), (20, 4099, 4100), (32, 20_001, 20_032),
                                    (33, 1531, 1600), (64, 70_001, 70_016), (64, 70_001, 70_003), (64, 63, 64),
                                    (1, 100, 128)])
def test_rows_with_a_leading_dimension(svgd, n, D, ld, carry):
    """Particles stored ld >= D floats apart (svgd_*_ld): same results as the dense layout, and
    the floats between the rows are neither read (they hold NaN) nor written."""
    X0, G0 = _random_problem(n, D, 3 * n + D + ld, x_std=0.3)
    eps = 0.05
    Xb, X = _padded(X0, ld, float("nan"))
    Gb, G = _padded(G0, ld, float("nan"))
    Pb, PHI = _padded(torch.zeros_like(X0), ld, 7.0)
    ref = orc.step(X0.cpu().numpy(), G0.cpu().numpy(), eps)
    with svgd.Svgd(n, D, flags=svgd.FLAG_CARRY_GRAM if carry else 0) as eng:
        h_bw = eng.bandwidth(X)
        eng.phi(X, G, PHI)
        h, K = eng.get_last(n)
        assert h_bw == h
        assert abs(h - ref["h"]) / ref["h"] <= TOL_H
        assert np.abs(K - ref["K"]).max() <= TOL_K
        e = np.abs(PHI.cpu().numpy() - ref["phi"]).max() / np.abs(ref["phi"]).max()
        assert e <= TOL_PHI, f"phi {e:.3e}"
        for step in range(3):            # steps 1 and 2 use the carried sums when carry is set
            Xh = X.cpu().numpy()
            eng.step(X, G, eps)
            h, K = eng.get_last(n)
            r = orc.step(Xh, G0.cpu().numpy(), eps)
            assert abs(h - r["h"]) / r["h"] <= TOL_H, f"step {step}"
            assert np.abs(K - r["K"]).max() <= TOL_K, f"step {step}"
            assert_x_new(X.cpu().numpy(), r, eps, f"step {step}")
    if ld > D:
        assert torch.isnan(Xb[:, D:]).all() and torch.isnan(Gb[:, D:]).all(), "padding of X or G was written"
        assert torch.all(Pb[:, D:] == 7.0), "padding of PHI was written"


def test_mixed_leading_dimensions_are_rejected(svgd):
    X = torch.zeros(4, 128, device="cuda")[:, :100]
    G = torch.zeros(4, 100, device="cuda")
    with svgd.Svgd(4, 100) as eng:
        with pytest.raises(ValueError):
            eng.step(X, G, 0.1)
        with pytest.raises(TypeError):
            eng.step(torch.zeros(100, 4, device="cuda").t(), G, 0.1)      # rows not contiguous
    lib = svgd._lib
    eng = svgd.Svgd(4, 100)
    assert lib.svgd_step_ld(eng._h, X.data_ptr(), G.data_ptr(), 4, 100, 99, 0.1, None) == -1   # ld < D
    eng.close()


@pytest.mark.parametrize("n,D,carry,padded", [(3, 800_000_001, True, False), (16, 150_000_001, False, False),
                                              (64, 34_000_001, True, False), (64, 34_000_001, True, True)])
def test_more_than_2_to_31_elements(svgd, n, D, carry, padded):
    """n * D = 2.4e9 elements (9.6 GB per array): element offsets beyond 32 bits on the vector-ALU
    and on the matrix-core path, dense rows and rows padded to 128 bytes.  h and K against the
    oracle's full pass; phi on column chunks at both ends and around element offset 2^31 (normalised
    by the oracle's maximum over those chunks); the in-place update == fl32(x + eps * phi_gpu) to one
    ulp on ALL entries, for the first step and (carry) for the second, which runs on carried sums."""
    assert n * D > 2 ** 31
    chunk = 4096
    g = torch.Generator(device="cuda")
    g.manual_seed(5 * n + 1)
    X = torch.randn(n, D, generator=g, device="cuda") * 0.02
    G = torch.randn(n, D, generator=g, device="cuda") * 1e-3
    if padded:
        Xd, Gd = X, G
        X, G = padded_copy(svgd, Xd), padded_copy(svgd, Gd)
        del Xd, Gd
        PHI = svgd.padded_rows(n, D)
    else:
        PHI = torch.empty_like(X)
    eps = 1e-3
    cross = (2 ** 31) % D   # a column at which some row's element offset passes 2^31
    starts = sorted({0, D - chunk, min(max(cross - chunk // 2, 0), D - chunk), D // 2 + 7})
    G_chunks = {s0: G[:, s0:s0 + chunk].cpu().numpy() for s0 in starts}

    def check_phi_chunks(Xh, h_ref, K_ref, what):
        refs = {s0: orc.phi_cols(np.ascontiguousarray(Xh[:, s0:s0 + chunk]), G_chunks[s0], K_ref, h_ref, 0, chunk)
                for s0 in starts}
        scale = max(float(np.abs(r).max()) for r in refs.values())
        for s0, ref in refs.items():
            got = PHI[:, s0:s0 + chunk].cpu().numpy().astype(np.float64)
            assert np.abs(got - ref).max() / scale <= TOL_PHI, f"{what}: chunk at {s0}"

    with svgd.Svgd(n, D, flags=svgd.FLAG_CARRY_GRAM if carry else 0) as eng, svgd.Svgd(n, D) as plain:
        X_old = X.clone()
        eng.phi(X, G, PHI)
        h, K = eng.get_last(n)
        eng.step(X, G, eps)
        Xh = X_old.cpu().numpy()
        h_ref, K_ref = oracle_kernel_matrix(Xh)
        assert abs(h - h_ref) / h_ref <= TOL_H, f"h {h} vs {h_ref}"
        assert np.abs(K - K_ref).max() <= TOL_K
        check_phi_chunks(Xh, h_ref, K_ref, "step 0")
        assert ulp_diff_device(X, X_old, PHI, eps) <= 1.0
        del Xh
        if carry:   # the next step takes its pair sums from the update that just ran
            X_old.copy_(X)
            plain.phi(X, G, PHI)
            eng.step(X, G, eps)
            h2, K2 = eng.get_last(n)
            X1h = X_old.cpu().numpy()
            h2_ref, K2_ref = oracle_kernel_matrix(X1h)
            assert abs(h2 - h2_ref) / h2_ref <= TOL_H
            assert np.abs(K2 - K2_ref).max() <= TOL_K
            check_phi_chunks(X1h, h2_ref, K2_ref, "step 1")
            assert ulp_diff_device(X, X_old, PHI, eps) <= 1.0


# ----------------------------------------------------------------------------------------------
# carried Gram (SVGD_FLAG_CARRY_GRAM): step t's update also accumulates the pair sums of the new
# X, and step t+1 skips its own pass over X
# ----------------------------------------------------------------------------------------------
@pytest.mark.parametrize("padded", [False, True])
@pytest.mark.parametrize("n,D", [(64, 70_001), (32, 4096), (17, 1531), (48, 129), (33, 200_000), (64, 63),
                                 (8, 100_003), (4, 1024), (16, 8577), (12, 70_001), (1, 100), (2, 65),
                                 (8, 3_000_017), (16, 70_001), (48, 20_011), (49, 5003), (64, 300_007), (12, 600_001)])
def test_carried_gram_matches_oracle_every_step(svgd, n, D, padded):
    """Four steps in a row with carried pair sums, on dense rows and on rows padded to 128 bytes
    (the layout that selects the direct-store instance of the matrix-core update kernel): h, K,
    phi against the oracle and X_new == fl32(x + eps * phi_gpu) to one ulp, every step.  Successive
    carried updates walk X in alternating directions, so steps 1 and 3 are backward walks and
    step 2 takes its h and K from the sums a backward walk left; the larger D give every
    wave several tiles (or every thread several column groups) in both directions."""
    X, G = _random_problem(n, D, 31 * n + D, x_std=0.3)
    check_carried_chain(svgd, X, G, 0.05, padded=padded, steps=4)


@pytest.mark.parametrize("padded", [False, True])
@pytest.mark.parametrize("D", [197, 300_007])
@pytest.mark.parametrize("n", [17, 18, 19, 20, 33, 34, 35, 36, 49, 50, 51, 52])
def test_particle_counts_just_above_a_multiple_of_16(svgd, n, D, padded):
    """One to four particles beyond a multiple of 16 are carried through the matrix-core update
    as remainder rows of the kernel for that multiple: a plain step (h, K, phi on all columns,
    in-place update to one ulp) and four carried steps (both walking directions, the remainder
    rows' pair sums feeding the next step's h and K), at a D with a few tiles in all and one that
    gives every wave several."""
    X, G = _random_problem(n, D, 7 * n + D, x_std=0.3)
    _plain_step_check(svgd, X, G, 0.05, padded=padded)
    check_carried_chain(svgd, X, G, 0.05, padded=padded, steps=4)


@pytest.mark.parametrize("n,D", [(16, 8577), (13, 4099), (24, 20_011), (32, 8577), (32, 4096), (17, 1531), (8, 100_003)])
def test_fused_single_launch_step_on_request(svgd, n, D):
    """SVGD_FLAG_FUSE_MFMA: with a short list of carried sums the step is one launch also on the
    matrix-core path (13 <= n <= 32) - seen in the launch counts - and its results match the oracle
    like every other path."""
    X, G = _random_problem(n, D, 7 * n + D, x_std=0.3)
    eps = 0.05
    with svgd.Svgd(n, D, flags=svgd.FLAG_CARRY_GRAM | svgd.FLAG_FUSE_MFMA) as eng:
        eng.step(X, G, eps)                   # pairwise-d2 pass, bandwidth, update
        eng.profile_begin()
        for step in range(3):                 # each of these: the update kernel alone
            Xh = X.cpu().numpy()
            eng.step(X, G, eps)
            h, K = eng.get_last(n)
            ref = orc.step(Xh, G.cpu().numpy(), eps)
            assert abs(h - ref["h"]) / ref["h"] <= TOL_H, f"step {step}"
            assert np.abs(K - ref["K"]).max() <= TOL_K, f"step {step}"
            assert_x_new(X.cpu().numpy(), ref, eps, f"step {step}")
        prof = eng.profile_end()
    assert [prof[k][1] for k in svgd.KERNEL_KINDS] == [0, 0, 0, 3]


def test_carried_gram_is_dropped_when_it_must_be(svgd):
    n, D = 32, 10_007
    X, G = _random_problem(n, D, 77)
    with svgd.Svgd(n, D, flags=svgd.FLAG_CARRY_GRAM) as eng:
        eng.step(X, G, 0.01)
        # the caller changes X behind the library's back and says so
        X.mul_(1.5)
        eng.forget_carry()
        Xh = X.cpu().numpy()
        eng.step(X, G, 0.01)
        h, _ = eng.get_last(n)
        assert abs(h - orc.step(Xh, G.cpu().numpy(), 0.01, want_phi=False, want_xnew=False)["h"]) / h <= TOL_H
        # a different buffer of the same shape is not mistaken for the carried one
        X2 = (X * 0.5).contiguous()
        X2h = X2.cpu().numpy()
        eng.step(X2, G, 0.01)
        h2, _ = eng.get_last(n)
        assert abs(h2 - orc.step(X2h, G.cpu().numpy(), 0.01, want_phi=False, want_xnew=False)["h"]) / h2 <= TOL_H
        # svgd_phi / svgd_bandwidth recompute from X and leave a consistent state behind
        PHI = torch.empty_like(X2)
        X2h = X2.cpu().numpy()
        eng.phi(X2, G, PHI)
        eng.step(X2, G, 0.01)
        h3, _ = eng.get_last(n)
        assert abs(h3 - orc.step(X2h, G.cpu().numpy(), 0.01, want_phi=False, want_xnew=False)["h"]) / h3 <= TOL_H


def test_carried_gram_is_dropped_on_another_stream(svgd):
    """The carried sums were written on the stream of the step that produced them; a step on another
    stream is not ordered behind that work, so it runs its own pass over X (seen as a launch of the
    pairwise-d2 kernel) - and its result is right."""
    n, D = 32, 50_021
    X, G = _random_problem(n, D, 78, x_std=0.3)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    with svgd.Svgd(n, D, flags=svgd.FLAG_CARRY_GRAM) as eng:
        torch.cuda.synchronize()
        eng.profile_begin()
        eng.step(X, G, 0.01, stream=s1)
        eng.step(X, G, 0.01, stream=s1)      # same stream: carried sums, no pass over X
        s1.synchronize()
        Xh = X.cpu().numpy()
        eng.step(X, G, 0.01, stream=s2)      # other stream: recomputed
        s2.synchronize()
        h, K = eng.get_last(n, stream=s2)
        prof = eng.profile_end()
    assert prof["gram"][1] == 2 and prof["update"][1] == 3
    ref = orc.step(Xh, G.cpu().numpy(), 0.01)
    assert abs(h - ref["h"]) / ref["h"] <= TOL_H
    assert np.abs(K - ref["K"]).max() <= TOL_K
    assert_x_new(X.cpu().numpy(), ref, 0.01)


@pytest.mark.parametrize("padded", [True, False])
@pytest.mark.parametrize("cfg_index", [3, 4, 5])
def test_full_size_carried_gram(svgd, cfg_index, padded):
    """Full-size configs in the launch configurations the benchmark times: pair sums carried from
    the previous update, rows padded to 128 bytes (the headline; at config 5 this is the instance
    update_mfma_kernel<4, false, true, true, true>) and dense rows.  Three steps: the first after
    a Gram pass, the second on carried sums and walking X backwards, the third on the sums that
    backward walk left; each step: h and K against the oracle, phi of ALL columns against the
    oracle at 1e-4 of max|phi|, X_new == fl32(x + eps * phi_gpu) to one ulp on all n * D entries."""
    wl = workloads.make(cfg_index, device="cuda")
    X0 = wl.X0
    G = wl.score(X0, 0)
    check_carried_chain(svgd, X0, G, wl.cfg.eps, padded=padded, steps=3)


@pytest.mark.parametrize("padded", [True, False])
@pytest.mark.parametrize("n,D", [(16, 9_000_001), (32, 4_400_003), (48, 3_000_001), (12, 12_000_001),
                                 (17, 5_000_003), (22, 4_000_001)])
def test_x_beyond_the_memory_side_cache(svgd, n, D, padded):
    """X of 550-580 MB at particle counts below 64: the sizes at which the pairwise-d2 pass visits
    the update's first tiles last (and streams the rest, on padded rows) and at which the workgroups
    of the matrix-core update on padded rows share a range; X of 340-350 MB at 17 and 22 particles:
    the sizes at which that update runs two workgroups per CU.  The plain step, then three steps on
    carried sums (forward, backward, forward), each checked completely against the oracle."""
    X0, G = _random_problem(n, D, 17 * n + 3, x_std=0.05)
    G *= 1e-2
    _plain_step_check(svgd, X0, G, 1e-3, padded=padded)
    check_carried_chain(svgd, X0, G, 1e-3, padded=padded, steps=3)


@pytest.mark.parametrize("seed", list(range(48)))
def test_random_shapes(svgd, seed):
    """Seeded random particle counts, lengths (log-uniform up to 400,000) and layouts: a plain step
    and three steps on carried sums, each checked completely against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.integers(1, 65))
    D = int(np.exp(rng.uniform(0.0, np.log(400_000.0))))
    padded = bool(rng.integers(0, 2))
    X0, G = _random_problem(n, D, 7 * seed + 1, x_std=float(rng.choice([0.02, 0.3, 1.0])))
    eps = float(rng.choice([1e-3, 0.05]))
    _plain_step_check(svgd, X0, G, eps, padded=padded)
    check_carried_chain(svgd, X0, G, eps, padded=padded, steps=3)


@pytest.mark.parametrize("n", [8, 20, 32, 33, 64])
@pytest.mark.parametrize("shift", [1, 3, 17])
def test_buffers_with_odd_base_alignment(svgd, n, shift):
    """X, G and PHI that start `shift` floats into their allocations (each with a different
    shift): the store windows of the update are aligned per row from the actual addresses."""
    D = 5003
    g = torch.Generator(device="cuda")
    g.manual_seed(n + shift)
    bufs = [torch.zeros(n * D + 64, device="cuda") for _ in range(3)]
    offs = [shift, shift + 2, shift + 5]
    X, G, PHI = [b[o:o + n * D].view(n, D) for b, o in zip(bufs, offs)]
    X.copy_(torch.randn(n, D, generator=g, device="cuda"))
    G.copy_(torch.randn(n, D, generator=g, device="cuda"))
    Xh, Gh = X.cpu().numpy(), G.cpu().numpy()
    ref = orc.step(Xh, Gh, 0.01)
    for flags in (0, svgd.FLAG_CARRY_GRAM):
        Xw = bufs[0].clone()[offs[0]:offs[0] + n * D].view(n, D)
        guard = Xw.storage_offset()
        with svgd.Svgd(n, D, flags=flags) as eng:
            eng.phi(Xw, G, PHI)
            eng.step(Xw, G, 0.01)
            eng.step(Xw, G, 0.0)     # second step (carried sums when flagged); eps = 0 leaves X as is
            torch.cuda.synchronize()
        e = np.abs(PHI.cpu().numpy() - ref["phi"]).max() / np.abs(ref["phi"]).max()
        assert e <= TOL_PHI
        assert_x_new(Xw.cpu().numpy(), ref, 0.01, f"flags={flags}")
        # nothing outside the n*D window was touched
        base = Xw._base if Xw._base is not None else Xw
        flat = base.view(-1)
        assert torch.all(flat[:guard] == 0) and torch.all(flat[guard + n * D:] == 0)
    assert torch.all(bufs[2][:offs[2]] == 0) and torch.all(bufs[2][offs[2] + n * D:] == 0)


@pytest.mark.parametrize("flags", [0, 1])
@pytest.mark.parametrize("n,D", [(4, 1024), (8, 4099), (32, 20_001)])
def test_step_can_be_captured_in_a_graph(svgd, n, D, flags):
    """svgd_step neither allocates nor synchronises, so a caller may capture it in a HIP graph.
    The graph is replayed several times with eager work and synchronisations in between, and
    every replay is compared with the same number of eager steps."""
    X0, G = _random_problem(n, D, 11 * n + flags, x_std=0.2)
    eps = 0.02
    # eager reference trajectory
    Xe = X0.clone()
    with svgd.Svgd(n, D, flags=flags) as eng:
        ref = []
        for _ in range(5):
            eng.step(Xe, G, eps)
            ref.append(Xe.clone())
    Xg = X0.clone()
    with svgd.Svgd(n, D, flags=flags) as eng:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            eng.step(Xg, G, eps, stream=side)          # warm-up on the capture stream (step 1)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eng.step(Xg, G, eps)                       # captured, not executed
        assert torch.equal(Xg, ref[0])
        for k in range(1, 5):
            graph.replay()
            torch.cuda.synchronize()
            junk = torch.randn(1000, device="cuda").sum().item()   # eager work between replays
            assert np.isfinite(junk)
            err = (Xg - ref[k]).abs().max().item() / ref[k].abs().max().item()
            assert err <= 1e-6, f"replay {k}: {err:.3e}"
