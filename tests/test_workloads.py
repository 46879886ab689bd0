"""The seeded input generator (inputs only: none of the method's arithmetic): the counter-based
definition pinned against a published test vector and a re-derivation in plain Python, torch and
numpy twins bit-identical, chunking irrelevant, distributions as stated."""
import math

import numpy as np
import torch

from paper_2306_06528_amd import workloads as w


def test_splitmix64_test_vector():
    # the first outputs of splitmix64 seeded with 0 (Steele, Lea & Flood; java.util.SplittableRandom)
    assert w._mix_int(0) == 0xE220A8397B1DCDAF
    assert w._mix_int(w._GAMMA) == 0x6E789E6AA1B965F4


def test_normal_is_the_stated_function_of_seed_array_and_index():
    seed, array_id = w.BASE_SEED + 5, 1
    base = w.stream_base(seed, array_id)
    got = w.normal_np(seed, array_id, 6)
    for e in range(6):
        bits = w._mix_int((base + e) & w._M64)
        u1 = ((bits >> 32) + 0.5) / 4294967296.0
        u2 = ((bits & 0xFFFFFFFF) + 0.5) / 4294967296.0
        want = np.float32(math.sqrt(-2.0 * math.log(u1)) * math.cos(2.0 * math.pi * u2))
        assert abs(float(got[e]) - float(want)) <= float(np.spacing(np.float32(abs(want))))


def test_torch_and_numpy_twins_agree_bit_for_bit():
    for seed, array_id, numel in ((1, 1, 1000), (w.BASE_SEED + 3, 2, 70_001)):
        assert np.array_equal(w.normal(seed, array_id, numel).numpy(), w.normal_np(seed, array_id, numel))
        assert np.array_equal(w.uniform(seed, array_id, numel).numpy(), w.uniform_np(seed, array_id, numel))


def test_chunking_does_not_matter(monkeypatch):
    a = w.normal(7, 3, 10_000)
    monkeypatch.setattr(w, "_CHUNK", 977)
    assert torch.equal(w.normal(7, 3, 10_000), a)
    assert torch.equal(w.normal(7, 3, 5000), a[:5000])


def test_streams_differ_and_distributions_are_as_stated():
    a, b = w.normal_np(11, 1, 200_000), w.normal_np(11, 2, 200_000)
    assert abs(float(np.corrcoef(a, b)[0, 1])) < 0.01
    assert abs(a.mean()) < 0.01 and abs(a.std() - 1.0) < 0.01
    u = w.uniform_np(11, 3, 200_000)
    assert 0.0 < u.min() and u.max() <= 1.0 and abs(u.mean() - 0.5) < 0.005
    wl = w.make(4, n=4, D=50_000)
    assert abs(float(wl.X0.std()) - 0.02) < 2e-4
    t = (wl.score(wl.X0) / 1e-3).numpy().ravel()
    assert abs(float(np.median(np.abs(t))) - 0.7649) < 0.01      # median |t(3)|


def test_configs_have_their_shapes():
    wl = w.make(2)
    assert wl.X0.shape == (16, 8577) and wl.score(wl.X0).shape == (16, 8577)
    assert torch.count_nonzero(wl.X0[:, 128:192]) == 0            # first layer's biases
    wl = w.make(3, n=4, D=1000)
    assert not torch.equal(wl.score(wl.X0, 0), wl.score(wl.X0, 1))   # redrawn every step
    assert torch.equal(wl.score(wl.X0, 1), wl.score(wl.X0, 1))
