"""How a PyTorch training loop uses the library without flattening anything per step.

The paper's routine (App. B.2) gathers, for every particle, a fresh flat copy of its parameters and
of their gradients.  Here the n x D matrices X and G exist once; every particle's nn.Module
parameters are views into its row of X and their .grad fields are views into the same row of G, so
autograd writes the scores straight into G and svgd_step moves the networks' weights in place.
The test trains n small MLPs on a synthetic regression task and checks each step against the
oracle.
"""
import numpy as np
import pytest
import torch

from oracle import svgd_oracle as orc
from parity_checks import assert_x_new

pytestmark = pytest.mark.gpu

TOL_H = 1e-5
TOL_K = 1e-5


def _make_particles(n, X, G, seed, width):
    """n MLPs whose parameters (and gradients) alias rows of X (and G)."""
    nets = []
    for i in range(n):
        torch.manual_seed(seed + i)
        net = torch.nn.Sequential(torch.nn.Linear(2, width), torch.nn.Tanh(),
                                  torch.nn.Linear(width, width), torch.nn.Tanh(),
                                  torch.nn.Linear(width, 1)).cuda()
        off = 0
        for p in net.parameters():
            k = p.numel()
            X[i, off:off + k].copy_(p.data.reshape(-1))
            p.data = X[i, off:off + k].view(p.shape)
            p.grad = G[i, off:off + k].view(p.shape)
            off += k
        assert off == X.shape[1]
        nets.append(net)
    return nets


# width 16: D = 337, the single-launch path; width 64: D = 4417, the multi-kernel path
@pytest.mark.parametrize("width", [16, 64])
def test_modules_as_views_of_the_particle_matrix(width):
    from paper_2306_06528_amd import svgd
    n = 6
    D = (2 * width + width) + (width * width + width) + (width + 1)
    # rows 128-byte aligned (the layout the kernels like best); the modules do not care
    X = svgd.padded_rows(n, D)
    G = svgd.padded_rows(n, D, fill=0.0)
    nets = _make_particles(n, X, G, seed=100, width=width)
    gen = torch.Generator(device="cuda").manual_seed(7)
    xs = torch.rand(256, 2, device="cuda", generator=gen) * 2 - 1
    ys = torch.sin(3 * xs[:, :1]) * xs[:, 1:]

    def log_posterior(net):          # Gaussian likelihood (sigma = 1) and N(0, 1) prior
        ll = -0.5 * ((net(xs) - ys) ** 2).sum()
        lp = -0.5 * sum((p ** 2).sum() for p in net.parameters())
        return ll + lp

    eps = 2e-4
    first = last = None
    with svgd.Svgd(n, D) as eng:
        for step in range(60):
            G.zero_()
            total = 0.0
            for net in nets:
                lp = log_posterior(net)
                lp.backward()        # accumulates the score into the row of G, in place
                total += lp.item()
            for net in nets:         # the gradients are still the views handed out above
                for p in net.parameters():
                    assert G.data_ptr() <= p.grad.data_ptr() < G.data_ptr() + n * G.stride(0) * 4
            first = total if first is None else first
            last = total
            Xh, Gh = X.cpu().numpy(), G.cpu().numpy()
            eng.step(X, G, eps)
            h, K = eng.get_last(n)
            ref = orc.step(Xh, Gh, eps)
            assert abs(h - ref["h"]) / ref["h"] <= TOL_H, f"step {step}"
            assert np.abs(K - ref["K"]).max() <= TOL_K, f"step {step}"
            assert_x_new(X.cpu().numpy(), ref, eps, f"step {step}")
    # the networks saw the update: their parameters are X, and the posterior went up
    for i, net in enumerate(nets):
        flat = torch.cat([p.data.reshape(-1) for p in net.parameters()])
        assert torch.equal(flat, X[i])
    assert last > first
    # the particles have not collapsed onto one another
    assert torch.cdist(X.contiguous(), X.contiguous()).fill_diagonal_(float("inf")).min().item() > 1e-3
