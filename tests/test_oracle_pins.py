"""Pins for the fp64 CPU oracle: closed forms, hand-worked values, library routines,
invariants and brute force.  CPU only.

Each pin is a function of a `step(X, G, eps) -> dict(d2, K, r, h, phi, X_new)` callable, so the
same pins are run (a) on the oracle, where all must hold, and (b) on deliberately wrong variants
of the method written here in numpy, where at least one pin must fail for each planted mistake.
"""
import math
import os

import numpy as np
import pytest
import scipy.spatial.distance as ssd
from sklearn.metrics.pairwise import rbf_kernel

from oracle import svgd_oracle as orc
from paper_2306_06528_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def oracle_step(X, G, eps):
    return orc.step(np.asarray(X), np.asarray(G), eps)


# ----------------------------------------------------------------------------------------------
# pins
# ----------------------------------------------------------------------------------------------
def _rng(seed):
    return np.random.default_rng(seed)


def pin_golden_two_particles(step):
    """Hand-worked n=2 example (tests/golden/two_particles.txt; App. B.2 routine, h = 2 l^2)."""
    vals = {}
    for line in open(os.path.join(GOLDEN, "two_particles.txt")):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        vals[k] = float(v)
    X = np.array([[0.0, 0.0], [3.0, 4.0]])
    G = np.array([[1.0, 0.0], [0.0, -2.0]])
    s = step(X, G, 0.5)
    assert s["d2"][0, 1] == pytest.approx(vals["d2_12"], rel=1e-14)
    assert s["h"] == pytest.approx(vals["h"], rel=1e-13)
    assert s["K"][0, 1] == pytest.approx(vals["K_12"], rel=1e-13)
    assert s["K"][1, 0] == pytest.approx(vals["K_12"], rel=1e-13)
    assert s["r"][0] == pytest.approx(vals["r_1"], rel=1e-13)
    want_phi = np.array([[vals["phi_1_x"], vals["phi_1_y"]], [vals["phi_2_x"], vals["phi_2_y"]]])
    want_x = np.array([[vals["x1_new_x"], vals["x1_new_y"]], [vals["x2_new_x"], vals["x2_new_y"]]])
    np.testing.assert_allclose(s["phi"], want_phi, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(s["X_new"], want_x, rtol=1e-12, atol=1e-14)


def pin_n2_kernel_is_one_ninth(step):
    """n=2: med over {0,0,d2,d2} = d2/2, h = d2/(2 ln 3), so K_12 = 3^-2 whatever the points."""
    r = _rng(1)
    for D in (1, 3, 50):
        X = r.normal(size=(2, D)) * 3.0
        G = r.normal(size=(2, D))
        s = step(X, G, 0.1)
        d2 = float(((X[0] - X[1]) ** 2).sum())
        assert s["h"] == pytest.approx(d2 / (2 * math.log(3)), rel=1e-13)
        assert s["K"][0, 1] == pytest.approx(1.0 / 9.0, rel=1e-12)


def pin_n2_repulsion_moves_apart(step):
    """G=0, n=2: each particle moves away from the other by (eps/2)(2/h)(1/9)|x_1-x_2|."""
    X = np.array([[1.0, 2.0, -1.0], [2.0, 0.0, 1.0]])
    G = np.zeros_like(X)
    eps = 0.3
    s = step(X, G, eps)
    diff = X[0] - X[1]
    dist = np.linalg.norm(diff)
    h = dist ** 2 / (2 * math.log(3))
    move = (eps / 2) * (2 / h) * (1 / 9)
    np.testing.assert_allclose(s["X_new"][0] - X[0], move * diff, rtol=1e-12)
    np.testing.assert_allclose(s["X_new"][1] - X[1], -move * diff, rtol=1e-12)
    assert np.linalg.norm(s["X_new"][0] - s["X_new"][1]) > dist


def pin_equidistant_closed_form(step):
    """x_i = a e_i: K_ij = 1/(n+1), r_i = 2n/(n+1), phi in closed form (golden/equidistant.txt)."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "equidistant.txt"))
            if l.strip() and not l.startswith("#")]
    r = _rng(2)
    for n_s, k_s, r_s in rows:
        n, k_off, r_i = int(n_s), float(k_s), float(r_s)
        a = 1.7
        D = n + 2
        X = np.zeros((n, D))
        X[np.arange(n), np.arange(n)] = a
        G = r.normal(size=(n, D))
        s = step(X, G, 0.01)
        off = ~np.eye(n, dtype=bool)
        np.testing.assert_allclose(s["d2"][off], 2 * a * a, rtol=1e-14)
        assert s["h"] == pytest.approx(2 * a * a / math.log(n + 1), rel=1e-13)
        np.testing.assert_allclose(s["K"][off], k_off, rtol=1e-12)
        np.testing.assert_allclose(np.diag(s["K"]), 1.0, rtol=0, atol=0)
        np.testing.assert_allclose(s["r"], r_i, rtol=1e-12)
        h = s["h"]
        want = np.empty_like(X)
        for i in range(n):
            others = [j for j in range(n) if j != i]
            want[i] = (G[i] + k_off * G[others].sum(0)
                       + (2 / h) * k_off * ((n - 1) * X[i] - X[others].sum(0))) / n
        np.testing.assert_allclose(s["phi"], want, rtol=1e-11, atol=1e-14)


def pin_d2_against_library_and_translation(step):
    """d2 equals scipy's squared-Euclidean cdist; unchanged by a common translation."""
    r = _rng(3)
    X = r.normal(size=(7, 33))
    G = r.normal(size=(7, 33))
    s = step(X, G, 0.1)
    np.testing.assert_allclose(s["d2"], ssd.cdist(X, X, "sqeuclidean"), rtol=1e-12, atol=1e-13)
    assert np.all(np.diag(s["d2"]) == 0.0)
    t = r.normal(size=(1, 33)) * 0.5
    s2 = step(X + t, G, 0.1)
    np.testing.assert_allclose(s2["d2"], s["d2"], rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(s2["phi"], s["phi"], rtol=1e-9, atol=1e-12)


def pin_median_and_kernel_against_library(step):
    """med = numpy.median over the full n x n matrix; K = sklearn rbf_kernel(gamma=1/h)."""
    r = _rng(4)
    for n in (3, 4, 5, 6, 9, 16):
        X = r.normal(size=(n, 12))
        G = r.normal(size=(n, 12))
        s = step(X, G, 0.1)
        med = float(np.median(ssd.cdist(X, X, "sqeuclidean")))
        assert s["h"] == pytest.approx(med / math.log(n + 1), rel=1e-12)
        np.testing.assert_allclose(s["K"], rbf_kernel(X, gamma=1.0 / s["h"]), rtol=1e-10)
        np.testing.assert_allclose(s["r"], s["K"].sum(1), rtol=1e-13)
        assert np.array_equal(s["K"], s["K"].T)
        assert np.all(np.diag(s["K"]) == 1.0)
        assert np.all((s["K"] > 0) & (s["K"] <= 1))
        if n % 2 == 0:
            # even n: order statistics n(n-2)/4 - 1 and n(n-2)/4 of the sorted pair distances
            pairs = np.sort(ssd.pdist(X, "sqeuclidean"))
            q = n * (n - 2) // 4
            assert med == pytest.approx(0.5 * (pairs[q - 1] + pairs[q]), rel=1e-13)


def pin_single_particle_is_gradient_ascent(step):
    """n=1: h falls back to 1, K=[1], phi = g, x <- x + eps g."""
    r = _rng(5)
    X = r.normal(size=(1, 9))
    G = r.normal(size=(1, 9))
    s = step(X, G, 0.25)
    assert s["h"] == 1.0
    assert s["K"].tolist() == [[1.0]]
    np.testing.assert_allclose(s["phi"], G, rtol=1e-15)
    np.testing.assert_allclose(s["X_new"], X + 0.25 * G, rtol=1e-15)


def pin_coincident_particles(step):
    """All particles equal: med = 0 -> h = 1, K = 1, phi_i = mean_j g_j."""
    r = _rng(6)
    x = r.normal(size=(1, 5))
    X = np.repeat(x, 4, axis=0)
    G = r.normal(size=(4, 5))
    s = step(X, G, 0.1)
    assert s["h"] == 1.0
    np.testing.assert_allclose(s["K"], 1.0)
    np.testing.assert_allclose(s["phi"], np.repeat(G.mean(0, keepdims=True), 4, 0), rtol=1e-14)


def pin_repulsion_sums_to_zero_and_permutation(step):
    """sum_i [n phi_i - sum_j K_ij g_j] = 0 (K symmetric); permuting particles permutes phi."""
    r = _rng(7)
    n, D = 6, 21
    X = r.normal(size=(n, D))
    G = r.normal(size=(n, D))
    s = step(X, G, 0.1)
    rep = n * s["phi"] - s["K"] @ G
    assert np.abs(rep).max() > 1e-3          # the repulsive term is really there
    np.testing.assert_allclose(rep.sum(0), 0.0, atol=1e-13)
    perm = r.permutation(n)
    sp = step(X[perm], G[perm], 0.1)
    np.testing.assert_allclose(sp["phi"], s["phi"][perm], rtol=1e-12, atol=1e-15)
    assert sp["h"] == pytest.approx(s["h"], rel=1e-14)


def pin_brute_force_per_pair(step):
    """phi by literal loops over (i, j, k) with k_ij recomputed per pair, as the paper's routine
    visits pairs (App. B.2), given only h from the n^2-entry median."""
    r = _rng(8)
    for n, D in ((2, 1), (3, 4), (5, 7), (4, 2)):
        X = r.normal(size=(n, D))
        G = r.normal(size=(n, D))
        eps = 0.07
        s = step(X, G, eps)
        allent = sorted(sum((X[i][k] - X[j][k]) ** 2 for k in range(D))
                        for i in range(n) for j in range(n))
        m = n * n
        med = allent[m // 2] if m % 2 else 0.5 * (allent[m // 2 - 1] + allent[m // 2])
        h = med / math.log(n + 1)
        assert s["h"] == pytest.approx(h, rel=1e-13)
        for i in range(n):
            for k in range(D):
                up = 0.0
                for j in range(n):
                    rad2 = sum((X[j][m_] - X[i][m_]) ** 2 for m_ in range(D))
                    kij = math.exp(-rad2 / h)
                    up += kij * G[j][k] + kij * (2.0 / h) * (X[i][k] - X[j][k])
                up /= n
                assert s["phi"][i, k] == pytest.approx(up, rel=1e-11, abs=1e-14)
                assert s["X_new"][i, k] == pytest.approx(X[i][k] + eps * up, rel=1e-13)


def pin_matrix_forms(step):
    """phi = (1/n)[K G + (2/h)(diag(r) X - K X)] (factored form) with library matmuls."""
    r = _rng(9)
    n, D = 8, 40
    X = r.normal(size=(n, D))
    G = r.normal(size=(n, D))
    s = step(X, G, 0.1)
    K, h = rbf_kernel(X, gamma=1.0 / s["h"]), s["h"]
    want = (K @ G + (2 / h) * (K.sum(1)[:, None] * X - K @ X)) / n
    np.testing.assert_allclose(s["phi"], want, rtol=1e-10, atol=1e-13)


def pin_gaussian_target_mean(step):
    """Config 1 (n=4, D=1024, N(mu, I) target, eps=0.05, 200 steps): the particle mean moves
    monotonically towards mu and ends within 0.05 sqrt(D) of it."""
    wl = workloads.make(1)
    X = wl.X0.double().numpy()
    mu = wl.mu.double().numpy()
    D = X.shape[1]
    err = [np.linalg.norm(X.mean(0) - mu)]
    for _ in range(wl.cfg.steps):
        G = -(X - mu)
        X = step(X, G, wl.cfg.eps)["X_new"]
        err.append(np.linalg.norm(X.mean(0) - mu))
    assert all(b < a for a, b in zip(err, err[1:]))
    assert err[-1] / math.sqrt(D) <= 0.05
    assert err[-1] < 0.1 * err[0]


PINS = [
    pin_golden_two_particles,
    pin_n2_kernel_is_one_ninth,
    pin_n2_repulsion_moves_apart,
    pin_equidistant_closed_form,
    pin_d2_against_library_and_translation,
    pin_median_and_kernel_against_library,
    pin_single_particle_is_gradient_ascent,
    pin_coincident_particles,
    pin_repulsion_sums_to_zero_and_permutation,
    pin_brute_force_per_pair,
    pin_matrix_forms,
    pin_gaussian_target_mean,
]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_pin(pin):
    pin(oracle_step)


def test_oracle_fp32_inputs_are_widened():
    """fp32 inputs give the same result as the same values passed as fp64."""
    r = _rng(10)
    X = r.normal(size=(5, 17)).astype(np.float32)
    G = r.normal(size=(5, 17)).astype(np.float32)
    a = orc.step(X, G, 0.1)
    b = orc.step(X.astype(np.float64), G.astype(np.float64), 0.1)
    for k in ("d2", "K", "r", "phi", "X_new"):   # threads may combine partial sums in any order
        np.testing.assert_allclose(a[k], b[k], rtol=1e-13, atol=1e-15)
    assert a["h"] == pytest.approx(b["h"], rel=1e-13)


def test_oracle_phi_cols_matches_full():
    r = _rng(11)
    X = r.normal(size=(6, 50)).astype(np.float32)
    G = r.normal(size=(6, 50)).astype(np.float32)
    s = orc.step(X, G, 0.1)
    part = orc.phi_cols(X, G, s["K"], s["h"], 13, 20)
    assert np.array_equal(part, s["phi"][:, 13:33])


# ----------------------------------------------------------------------------------------------
# planted mistakes: a numpy re-statement of the method with one switchable error each.  None of
# these is used to produce expected values; they only show that the pins above have teeth.
# ----------------------------------------------------------------------------------------------
MUTATIONS = [
    "attract",            # kernel-gradient term with the wrong sign
    "no_two",             # 1/h instead of 2/h
    "log_n",              # ln(n) instead of ln(n+1)
    "median_upper",       # median over the strict upper triangle only
    "median_low",         # lower middle instead of mean-of-middle for even counts
    "no_self",            # j = i left out of the sum
    "div_n_minus_1",      # 1/(n-1) instead of 1/n
    "K_transposed_grad",  # uses g_i instead of g_j in the driving term
    "gauss_seidel",       # particles updated one after the other
    "half_h",             # K = exp(-d2/(2h))
    "descent",            # x <- x - eps phi
    "sqrt_dist",          # median of distances instead of squared distances
    "no_guard",           # h = 0 not replaced
    "drop_drive",         # driving term missing
]


def mutant_step(mut):
    def step(X, G, eps):
        X = np.asarray(X, np.float64)
        G = np.asarray(G, np.float64)
        n = X.shape[0]

        def kern(Xc):
            d2 = ((Xc[:, None, :] - Xc[None, :, :]) ** 2).sum(-1)
            base = np.sqrt(d2) if mut == "sqrt_dist" else d2
            if mut == "median_upper":
                vals = base[np.triu_indices(n, 1)]
                med = np.median(vals) if vals.size else 0.0
            elif mut == "median_low":
                med = np.sort(base.ravel())[(n * n - 1) // 2]
            else:
                med = np.median(base)
            with np.errstate(divide="ignore", invalid="ignore"):
                h = med / (math.log(n) if mut == "log_n" else math.log(n + 1))
            if mut != "no_guard" and not (h > 0):
                h = 1.0
            with np.errstate(divide="ignore", invalid="ignore"):
                K = np.exp(-d2 / (2 * h if mut == "half_h" else h))
            return d2, h, K

        d2, h, K = kern(X)
        coef = (1.0 if mut == "no_two" else 2.0) / h
        sign = -1.0 if mut == "attract" else 1.0
        Xc = X.copy()
        phi = np.zeros_like(X)
        for i in range(n):
            if mut == "gauss_seidel":
                _, h_i, K_i = kern(Xc)
            else:
                K_i = K
            acc = np.zeros(X.shape[1])
            for j in range(n):
                if mut == "no_self" and j == i:
                    continue
                gj = G[i] if mut == "K_transposed_grad" else G[j]
                drive = 0.0 if mut == "drop_drive" else K_i[i, j] * gj
                acc += drive + sign * coef * K_i[i, j] * (Xc[i] - Xc[j])
            phi[i] = acc / ((n - 1) if (mut == "div_n_minus_1" and n > 1) else n)
            if mut == "gauss_seidel":
                Xc[i] = Xc[i] + eps * phi[i]
        X_new = X + (-eps if mut == "descent" else eps) * phi
        return dict(d2=d2, K=K, r=K.sum(1), h=h, phi=phi, X_new=X_new)
    return step


def test_unmutated_restatement_passes_all_pins():
    """Sanity of the mutation harness itself: with no mistake planted every pin holds."""
    for pin in PINS:
        pin(mutant_step(None))


@pytest.mark.parametrize("mut", MUTATIONS)
def test_pins_catch_planted_mistake(mut):
    caught = []
    for pin in PINS:
        if pin is pin_gaussian_target_mean:
            continue  # slow in numpy; the cheap pins must do the catching
        try:
            with np.errstate(all="ignore"):
                pin(mutant_step(mut))
        except (AssertionError, FloatingPointError, ValueError, ZeroDivisionError):
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake {mut!r}"


# ----------------------------------------------------------------------------------------------
# the fixed-bandwidth mode (the paper's own kernel, App. B.2: k = exp(-|.|^2 / (2 l^2)), h = 2 l^2)
# ----------------------------------------------------------------------------------------------
def test_fixed_bandwidth_matches_library_kernel():
    r = _rng(21)
    X, G = r.normal(size=(7, 11)), r.normal(size=(7, 11))
    ell = 1.7
    s = orc.step(X, G, 0.1, h_fixed=2 * ell * ell)
    assert s["h"] == 2 * ell * ell
    np.testing.assert_allclose(s["K"], rbf_kernel(X, gamma=1.0 / (2 * ell * ell)), rtol=1e-13)
    # phi from the definition, pair by pair
    n = 7
    want = np.zeros_like(X)
    for i in range(n):
        for j in range(n):
            want[i] += s["K"][i, j] * G[j] + (2.0 / s["h"]) * s["K"][i, j] * (X[i] - X[j])
    np.testing.assert_allclose(s["phi"], want / n, rtol=1e-12)


def test_fixed_bandwidth_limits():
    """h -> infinity: K -> 1 and phi_i -> mean_j g_j;  h -> 0: K -> I and phi_i -> g_i / n."""
    r = _rng(22)
    X, G = r.normal(size=(5, 8)), r.normal(size=(5, 8))
    s = orc.step(X, G, 0.1, h_fixed=1e30)
    np.testing.assert_allclose(s["K"], 1.0, rtol=0, atol=1e-15)
    np.testing.assert_allclose(s["phi"], np.repeat(G.mean(0, keepdims=True), 5, 0), rtol=1e-12)
    s = orc.step(X, G, 0.1, h_fixed=1e-30)
    np.testing.assert_array_equal(s["K"], np.eye(5))
    np.testing.assert_allclose(s["phi"], G / 5, rtol=1e-15)
