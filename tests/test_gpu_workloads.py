"""The input generator gives the same buffers on the GPU as on the CPU: the integer part exactly,
the fp64 Box-Muller step up to the last bit of the device's log and cos before the one rounding
to fp32."""
import numpy as np
import pytest
import torch

from paper_2306_06528_amd import workloads as w

pytestmark = pytest.mark.gpu


def test_bits_and_uniforms_are_identical_on_both_devices():
    base = w.stream_base(w.BASE_SEED + 5, 1)
    assert torch.equal(w._bits_torch(base, 12345, 100_000, "cuda").cpu(), w._bits_torch(base, 12345, 100_000, "cpu"))
    assert torch.equal(w.uniform(9, 3, 300_001, "cuda").cpu(), w.uniform(9, 3, 300_001))


def test_normals_agree_with_the_numpy_twin_to_one_rounding():
    numel = (1 << 22) + 4097                       # crosses a chunk boundary
    a = w.normal(w.BASE_SEED + 4, 1, numel, "cuda").cpu().numpy()
    b = w.normal_np(w.BASE_SEED + 4, 1, numel)
    differ = a != b
    assert differ.mean() < 1e-4                    # only where fp64 rounding straddles an fp32 tie
    assert np.all(np.abs(a[differ] - b[differ]) <= np.spacing(np.abs(b[differ])))


def test_a_workload_is_the_same_on_both_devices():
    g, c = w.make(3, device="cuda", n=5, D=70_001), w.make(3, n=5, D=70_001)
    torch.testing.assert_close(g.X0.cpu(), c.X0, rtol=2e-7, atol=0)
    torch.testing.assert_close(g.score(g.X0, 2).cpu(), c.score(c.X0, 2), rtol=1e-5, atol=1e-9)
