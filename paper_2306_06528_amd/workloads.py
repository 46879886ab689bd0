"""Seeded synthetic particle workloads (inputs only; none of the SVGD arithmetic).

Each workload stands in for one of the paper's particle populations (Sec. 5.1 and
App. C: NN particles of 1..32 networks per run): only the particle count n and the
flattened parameter count D matter to the all-particle update, so X is drawn with
the value distribution a freshly initialised network of that size has, and the
score G = grad log p(x) comes from a synthetic target.

Generation uses torch's seeded generators on the requested device; a workload is
generated once and the same buffers are handed to every consumer.
"""
from dataclasses import dataclass
from typing import Optional

import torch

BASE_SEED = 230606528


@dataclass(frozen=True)
class Config:
    index: int            # 1-based
    name: str
    n: int
    D: int
    eps: float
    steps: int
    x_kind: str           # "normal" | "mlp"
    x_std: float
    g_kind: str           # "gauss_iso" | "gauss_diag" | "gauss_iso_noisy" | "student_t"


CONFIGS = {
    1: Config(1, "tiny", 4, 1024, 0.05, 200, "normal", 1.0, "gauss_iso"),
    2: Config(2, "pinn_mlp", 16, 8577, 1e-3, 1000, "mlp", 0.0, "gauss_diag"),
    3: Config(3, "operator_net", 32, 2_000_000, 1e-4, 50, "normal", 0.05, "gauss_iso_noisy"),
    4: Config(4, "resnet18", 8, 11_173_962, 1e-4, 20, "normal", 0.02, "student_t"),
    5: Config(5, "large_ensemble", 64, 11_173_962, 1e-4, 10, "normal", 0.02, "student_t"),
}

# flattened 2-64-64-64-1 tanh MLP: [W1,b1,W2,b2,W3,b3,W4,b4]
_MLP_LAYERS = [(2, 64), (64, 64), (64, 64), (64, 1)]


class Workload:
    """X0 and a score function for one config.  `score(X, step)` returns G for the given X."""

    def __init__(self, cfg: Config, device="cpu", n: Optional[int] = None, D: Optional[int] = None):
        self.cfg = cfg
        self.n = cfg.n if n is None else n
        self.D = cfg.D if D is None else D
        self.device = torch.device(device)
        self.seed = BASE_SEED + cfg.index
        self._gen = torch.Generator(device=self.device)
        self._gen.manual_seed(self.seed)
        n_, D_ = self.n, self.D
        if cfg.x_kind == "normal":
            self.X0 = self._randn(n_, D_) * cfg.x_std
        else:
            if D_ != 8577:
                raise ValueError("the MLP layout has D = 8577")
            parts = []
            for fan_in, fan_out in _MLP_LAYERS:
                parts.append(self._randn(n_, fan_in * fan_out) * (1.0 / fan_in) ** 0.5)
                parts.append(torch.zeros(n_, fan_out, device=self.device))
            self.X0 = torch.cat(parts, dim=1).contiguous()
        self.mu = None
        self.inv_sigma2 = None
        self._G_fixed = None
        if cfg.g_kind == "gauss_iso":
            self.mu = self._randn(D_)
        elif cfg.g_kind == "gauss_diag":
            self.mu = self._randn(D_)
            sigma = 0.5 + 1.5 * torch.rand(D_, generator=self._gen, device=self.device)
            self.inv_sigma2 = 1.0 / (sigma * sigma)
        elif cfg.g_kind == "gauss_iso_noisy":
            self.mu = self._randn(D_) * 0.05
        elif cfg.g_kind == "student_t":
            z0 = self._randn(n_, D_)
            s = torch.zeros(n_, D_, device=self.device)
            for _ in range(3):
                z = self._randn(n_, D_)
                s.addcmul_(z, z)
                del z
            self._G_fixed = (z0 / torch.sqrt(s / 3.0) * 1e-3).contiguous()
            del z0, s
        else:
            raise ValueError(cfg.g_kind)

    def _randn(self, *shape):
        return torch.randn(*shape, generator=self._gen, device=self.device, dtype=torch.float32)

    def score(self, X: torch.Tensor, step: int = 0) -> torch.Tensor:
        """G = grad log p at X for this workload's synthetic target (fp32, same shape as X)."""
        kind = self.cfg.g_kind
        if kind == "student_t":
            return self._G_fixed
        if kind == "gauss_iso":
            return (self.mu - X).contiguous()
        if kind == "gauss_diag":
            return ((self.mu - X) * self.inv_sigma2).contiguous()
        g = torch.Generator(device=self.device)
        g.manual_seed(self.seed * 1000003 + step + 1)
        noise = torch.randn(X.shape, generator=g, device=self.device, dtype=torch.float32) * 1e-4
        return ((self.mu - X) + noise).contiguous()


def make(index: int, device="cpu", n: Optional[int] = None, D: Optional[int] = None) -> Workload:
    """Workload for benchmark configuration `index` (1..5); n/D override the size (distributions kept)."""
    return Workload(CONFIGS[index], device=device, n=n, D=D)
