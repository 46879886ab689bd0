"""Pins for the oracle's SWAG running moments (paper Sec. 2: first and second moments of the
parameter trajectory, per particle for multi-SWAG).  CPU only."""
import numpy as np
import pytest

from oracle import svgd_oracle as orc


def run(update, traj):
    mean = np.zeros_like(traj[0], dtype=np.float64)
    sq = np.zeros_like(mean)
    for t, x in enumerate(traj):
        update(mean, sq, x, t)
    return mean, sq


def oracle_update(mean, sq, x, count):
    orc.swag_update(mean, sq, np.ascontiguousarray(x), count)


def pin_moments_equal_library_means(update):
    """After T updates: mean = numpy.mean of the trajectory, sq = numpy.mean of its squares,
    sq - mean^2 = numpy.var (the diagonal SWAG covariance)."""
    r = np.random.default_rng(0)
    traj = r.normal(size=(17, 3, 11))
    mean, sq = run(update, list(traj))
    np.testing.assert_allclose(mean, traj.mean(0), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(sq, (traj ** 2).mean(0), rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(sq - mean ** 2, traj.var(0), rtol=1e-10, atol=1e-13)


def pin_first_update_copies_the_iterate(update):
    r = np.random.default_rng(1)
    x = r.normal(size=(2, 5))
    mean = np.full_like(x, 123.0)   # whatever was there is weighted by count = 0
    sq = np.full_like(x, -7.0)
    update(mean, sq, x, 0)
    np.testing.assert_allclose(mean, x, rtol=1e-15)
    np.testing.assert_allclose(sq, x * x, rtol=1e-15)


def pin_constant_trajectory(update):
    x = np.array([[1.5, -2.0, 0.25]])
    mean, sq = run(update, [x] * 9)
    np.testing.assert_allclose(mean, x, rtol=1e-15)
    np.testing.assert_allclose(sq, x * x, rtol=1e-15)


def pin_hand_worked(update):
    """x = 1, 2, 6 -> mean 1, 1.5, 3; squares 1, 4, 36 -> sq 1, 2.5, 41/3."""
    mean = np.zeros((1, 1)); sq = np.zeros((1, 1))
    for t, (x, m, s) in enumerate([(1.0, 1.0, 1.0), (2.0, 1.5, 2.5), (6.0, 3.0, 41.0 / 3.0)]):
        update(mean, sq, np.array([[x]]), t)
        assert mean[0, 0] == pytest.approx(m, rel=1e-15)
        assert sq[0, 0] == pytest.approx(s, rel=1e-15)


def pin_particles_are_independent(update):
    """multi-SWAG: row i of the moments depends on row i of the iterates only."""
    r = np.random.default_rng(2)
    traj = r.normal(size=(6, 4, 7))
    mean, sq = run(update, list(traj))
    traj2 = traj.copy()
    traj2[:, 2] += 5.0
    mean2, sq2 = run(update, list(traj2))
    keep = [0, 1, 3]
    np.testing.assert_array_equal(mean[keep], mean2[keep])
    np.testing.assert_array_equal(sq[keep], sq2[keep])
    assert not np.allclose(mean[2], mean2[2])


PINS = [pin_moments_equal_library_means, pin_first_update_copies_the_iterate, pin_constant_trajectory,
        pin_hand_worked, pin_particles_are_independent]


@pytest.mark.parametrize("pin", PINS, ids=lambda p: p.__name__)
def test_oracle_swag_pin(pin):
    pin(oracle_update)


def test_fp32_iterates_are_widened():
    r = np.random.default_rng(3)
    traj = r.normal(size=(5, 2, 9)).astype(np.float32)
    a = run(oracle_update, list(traj))
    b = run(oracle_update, list(traj.astype(np.float64)))
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])


MUTATIONS = ["divide_by_count", "no_square", "exponential_average", "weight_swapped", "sq_of_mean"]


def mutant(mut):
    def update(mean, sq, x, count):
        c = float(count)
        if mut == "divide_by_count":
            d = max(c, 1.0)
            mean[...] = (c * mean + x) / d
            sq[...] = (c * sq + x * x) / d
        elif mut == "no_square":
            mean[...] = (c * mean + x) / (c + 1)
            sq[...] = (c * sq + x) / (c + 1)
        elif mut == "exponential_average":
            mean[...] = 0.5 * mean + 0.5 * x
            sq[...] = 0.5 * sq + 0.5 * x * x
        elif mut == "weight_swapped":
            mean[...] = (mean + c * x) / (c + 1)
            sq[...] = (sq + c * x * x) / (c + 1)
        elif mut == "sq_of_mean":
            mean[...] = (c * mean + x) / (c + 1)
            sq[...] = mean * mean
    return update


@pytest.mark.parametrize("mut", MUTATIONS)
def test_pins_catch_planted_mistake(mut):
    caught = []
    for pin in PINS:
        try:
            pin(mutant(mut))
        except AssertionError:
            caught.append(pin.__name__)
    assert caught, f"no pin notices the planted mistake {mut!r}"
