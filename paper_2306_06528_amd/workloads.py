"""Seeded synthetic particle workloads (inputs only; none of the SVGD arithmetic).

Each workload stands in for one of the paper's particle populations (Sec. 5.1 and
App. C: NN particles of 1..32 networks per run): only the particle count n and the
flattened parameter count D matter to the all-particle update, so X is drawn with
the value distribution a freshly initialised network of that size has, and the
score G = grad log p(x) comes from a synthetic target.

Every number comes from a counter-based generator: element e of array a of a workload with
seed s is a pure function of (s, a, e) - splitmix64 of a stream base plus the element index, the
upper and lower 32 bits of the hash as two uniforms, Box-Muller for a normal variate - so the same
buffers are obtained on the CPU and on the GPU, in any chunking, and with numpy alone
(`normal_np`, `uniform_np`: the same arithmetic without torch).  Integer steps are exact; the
Box-Muller step runs in fp64 and is rounded to fp32 once.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np
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


# ---------------------------------------------------------------------------------------------
# the counter-based generator (splitmix64: Steele, Lea & Flood, "Fast splittable pseudorandom
# number generators", OOPSLA 2014 - the output function of SplittableRandom)
# ---------------------------------------------------------------------------------------------
_M64 = (1 << 64) - 1
_GAMMA = 0x9E3779B97F4A7C15
_MUL1 = 0xBF58476D1CE4E5B9
_MUL2 = 0x94D049BB133111EB


def _mix_int(z: int) -> int:
    """splitmix64 output function on a Python int (mod 2^64)."""
    z = (z + _GAMMA) & _M64
    z = ((z ^ (z >> 30)) * _MUL1) & _M64
    z = ((z ^ (z >> 27)) * _MUL2) & _M64
    return z ^ (z >> 31)


def stream_base(seed: int, array_id: int) -> int:
    """Where the counter of array `array_id` of the workload with `seed` starts (mod 2^64)."""
    return _mix_int((_mix_int(seed & _M64) + array_id) & _M64)


def _signed(v: int) -> int:
    return v - (1 << 64) if v >= (1 << 63) else v


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right of int64 bit patterns."""
    return (z >> k) & ((1 << (64 - k)) - 1)


def _bits_torch(base: int, start: int, count: int, device) -> torch.Tensor:
    """The hashes of elements start .. start+count-1 as int64 bit patterns (wrapping arithmetic)."""
    z = torch.arange(start, start + count, dtype=torch.int64, device=device) + _signed((base + _GAMMA) & _M64)
    z = (z ^ _lsr(z, 30)) * _signed(_MUL1)
    z = (z ^ _lsr(z, 27)) * _signed(_MUL2)
    return z ^ _lsr(z, 31)


def _uniforms_torch(bits: torch.Tensor):
    """(u1, u2) in (0, 1), fp64, from the upper and the lower 32 bits."""
    hi = _lsr(bits, 32).to(torch.float64)
    lo = (bits & 0xFFFFFFFF).to(torch.float64)
    return (hi + 0.5) * (1.0 / 4294967296.0), (lo + 0.5) * (1.0 / 4294967296.0)


# elements per batch of tensor operations: on the CPU what the caches like; on a GPU large, so that
# a big workload takes hundreds of kernel launches, not tens of thousands (a profiler that
# collects hardware counters instruments every launch)
_CHUNK = 1 << 22
_CHUNK_GPU = 1 << 27


def _chunk(device) -> int:
    return _CHUNK if torch.device(device).type == "cpu" else _CHUNK_GPU


def uniform(seed: int, array_id: int, numel: int, device="cpu") -> torch.Tensor:
    """numel uniforms in (0, 1), fp32 (the upper 32 bits of each hash)."""
    base = stream_base(seed, array_id)
    out = torch.empty(numel, dtype=torch.float32, device=device)
    step = _chunk(device)
    for s0 in range(0, numel, step):
        c = min(step, numel - s0)
        u1, _ = _uniforms_torch(_bits_torch(base, s0, c, device))
        out[s0:s0 + c] = u1.to(torch.float32)
    return out


def normal(seed: int, array_id: int, numel: int, device="cpu") -> torch.Tensor:
    """numel standard normal variates, fp32: sqrt(-2 ln u1) cos(2 pi u2) per element."""
    base = stream_base(seed, array_id)
    out = torch.empty(numel, dtype=torch.float32, device=device)
    step = _chunk(device)
    for s0 in range(0, numel, step):
        c = min(step, numel - s0)
        u1, u2 = _uniforms_torch(_bits_torch(base, s0, c, device))
        out[s0:s0 + c] = (torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * np.pi) * u2)).to(torch.float32)
    return out


def _bits_np(base: int, start: int, count: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        z = np.arange(start, start + count, dtype=np.uint64) + np.uint64((base + _GAMMA) & _M64)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(_MUL1)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(_MUL2)
        return z ^ (z >> np.uint64(31))


def uniform_np(seed: int, array_id: int, numel: int) -> np.ndarray:
    """`uniform` without torch."""
    bits = _bits_np(stream_base(seed, array_id), 0, numel)
    return (((bits >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)).astype(np.float32)


def normal_np(seed: int, array_id: int, numel: int) -> np.ndarray:
    """`normal` without torch."""
    bits = _bits_np(stream_base(seed, array_id), 0, numel)
    u1 = ((bits >> np.uint64(32)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    u2 = ((bits & np.uint64(0xFFFFFFFF)).astype(np.float64) + 0.5) * (1.0 / 4294967296.0)
    return (np.sqrt(-2.0 * np.log(u1)) * np.cos((2.0 * np.pi) * u2)).astype(np.float32)


# array ids within a workload's seed
_A_X0, _A_MU, _A_SIGMA, _A_T0 = 1, 2, 3, 4   # _A_T0 .. _A_T0 + 3: the four normals of a Student-t(3)
_A_MLP = 16                                   # + layer index
_A_NOISE = 1000                               # + step


class Workload:
    """X0 and a score function for one config.  `score(X, step)` returns G for the given X."""

    def __init__(self, cfg: Config, device="cpu", n: Optional[int] = None, D: Optional[int] = None):
        self.cfg = cfg
        self.n = cfg.n if n is None else n
        self.D = cfg.D if D is None else D
        self.device = torch.device(device)
        self.seed = BASE_SEED + cfg.index
        n_, D_ = self.n, self.D
        if cfg.x_kind == "normal":
            self.X0 = self._randn(_A_X0, n_, D_).mul_(cfg.x_std)
        else:
            if D_ != 8577:
                raise ValueError("the MLP layout has D = 8577")
            parts = []
            for layer, (fan_in, fan_out) in enumerate(_MLP_LAYERS):
                parts.append(self._randn(_A_MLP + layer, n_, fan_in * fan_out) * (1.0 / fan_in) ** 0.5)
                parts.append(torch.zeros(n_, fan_out, device=self.device))
            self.X0 = torch.cat(parts, dim=1).contiguous()
        self.mu = None
        self.inv_sigma2 = None
        self._G_fixed = None
        if cfg.g_kind == "gauss_iso":
            self.mu = self._randn(_A_MU, D_)
        elif cfg.g_kind == "gauss_diag":
            self.mu = self._randn(_A_MU, D_)
            sigma = 0.5 + 1.5 * uniform(self.seed, _A_SIGMA, D_, self.device)
            self.inv_sigma2 = 1.0 / (sigma * sigma)
        elif cfg.g_kind == "gauss_iso_noisy":
            self.mu = self._randn(_A_MU, D_) * 0.05
        elif cfg.g_kind == "student_t":
            # t(3) = Z0 / sqrt((Z1^2 + Z2^2 + Z3^2) / 3)
            s = torch.zeros(n_, D_, device=self.device)
            for k in range(1, 4):
                z = self._randn(_A_T0 + k, n_, D_)
                s.addcmul_(z, z)
                del z
            g = self._randn(_A_T0, n_, D_)
            g.div_(torch.sqrt(s.div_(3.0))).mul_(1e-3)
            self._G_fixed = g
            del s
        else:
            raise ValueError(cfg.g_kind)

    def _randn(self, array_id, *shape):
        numel = 1
        for d in shape:
            numel *= d
        return normal(self.seed, array_id, numel, self.device).view(*shape)

    def score(self, X: torch.Tensor, step: int = 0) -> torch.Tensor:
        """G = grad log p at X for this workload's synthetic target (fp32, same shape as X)."""
        kind = self.cfg.g_kind
        if kind == "student_t":
            return self._G_fixed
        if kind == "gauss_iso":
            return (self.mu - X).contiguous()
        if kind == "gauss_diag":
            return ((self.mu - X) * self.inv_sigma2).contiguous()
        noise = normal(self.seed, _A_NOISE + step, X.numel(), self.device).view(X.shape).mul_(1e-4)
        return ((self.mu - X) + noise).contiguous()


def make(index: int, device="cpu", n: Optional[int] = None, D: Optional[int] = None) -> Workload:
    """Workload for benchmark configuration `index` (1..5); n/D override the size (distributions kept)."""
    return Workload(CONFIGS[index], device=device, n=n, D=D)
