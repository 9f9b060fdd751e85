"""Seeded synthetic inputs for the CO3 codec: the only module shared by the CPU oracle's
tests and the GPU path's tests / bench.  It holds none of the codec's arithmetic: it draws
gradients, lays out layers (segments) and applies the workload's rule for the exponent bias.

The paper measures on CIFAR-10 training runs of three CNNs (Sec. II-C); their gradients are
not available here, so zero-location GenNorm vectors stand in for them: the density of
eq. (gennorm), shape beta < 2 and scale around 1e-3 as in the histograms of Sec. III, one
distribution per layer as assumed in Sec. II-D.  A GenNorm(0, alpha, beta) variate is
alpha * s * G^(1/beta) with s a random sign and G ~ Gamma(1/beta, 1).
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

SEED_BASE = 0xC03


def seed_for(cfg: int, it: int, user: int) -> int:
    return SEED_BASE ^ ((cfg << 20) + (it << 10) + user)


@dataclass
class Workload:
    name: str
    cfg: int
    U: int
    d: int
    E: int
    M: int
    gamma: float                       # memory-decay coefficient (lambda of the workload list)
    iters: int
    gammas: tuple = ()                 # every coefficient the workload names (default: just gamma)
    beta: Optional[float] = None       # None: per-user, uniform in beta_range
    beta_range: tuple = (0.6, 1.4)
    alpha: Optional[float] = None      # None: per-user log-uniform in alpha_range
    alpha_range: tuple = (1e-4, 1e-2)
    nseg: int = 1
    seg_alpha_range: Optional[tuple] = None   # per-segment scales, log-spaced then shuffled
    outlier_frac: float = 0.0
    outlier_scale: float = 1.0
    per_user_books: bool = False
    seg_len: List[int] = field(default_factory=list)

    def __post_init__(self):
        if not self.gammas:
            self.gammas = (self.gamma,)
        if not self.seg_len:
            self.seg_len = powerlaw_segments(self.d, self.nseg) if self.nseg > 1 else [self.d]

    def user_params(self, user: int):
        """(beta, alpha) of one user, fixed over iterations."""
        rng = np.random.default_rng(seed_for(self.cfg, 1023, user))
        beta = self.beta if self.beta is not None else float(rng.uniform(*self.beta_range))
        if self.alpha is not None:
            alpha = self.alpha
        else:
            lo, hi = np.log(self.alpha_range[0]), np.log(self.alpha_range[1])
            alpha = float(np.exp(rng.uniform(lo, hi)))
        return beta, alpha

    def seg_alphas(self):
        if self.seg_alpha_range is None:
            return None
        lo, hi = self.seg_alpha_range
        a = np.logspace(np.log10(lo), np.log10(hi), self.nseg)
        np.random.default_rng(seed_for(self.cfg, 1022, 0)).shuffle(a)
        return a

    def scaled(self, d: int, U: Optional[int] = None) -> "Workload":
        """Same recipe at another size (for parity tests the oracle finishes in seconds)."""
        w = Workload(**{**self.__dict__, "d": d, "U": self.U if U is None else U, "seg_len": []})
        return w


def powerlaw_segments(d: int, nseg: int, exponent: float = 1.2) -> List[int]:
    """Layer-shaped split: sizes proportional to (k+1)^-exponent, rounded, unaligned, sum d."""
    w = np.arange(1, nseg + 1, dtype=np.float64) ** (-exponent)
    sizes = np.floor(w / w.sum() * d).astype(np.int64)
    sizes |= 1                                   # odd: never a multiple of any tile
    sizes[0] += d - int(sizes.sum())
    assert sizes.min() > 0 and int(sizes.sum()) == d
    return [int(s) for s in sizes]


WORKLOADS = {
    "cfg1": Workload("cfg1", 1, U=1, d=1 << 20, E=3, M=0, gamma=0.9, iters=3, beta=1.0, alpha=1e-3),
    "cfg2": Workload("cfg2", 2, U=10, d=11_689_512, E=4, M=1, gamma=0.9, iters=5, beta=0.8, alpha=1e-3),
    "cfg3": Workload("cfg3", 3, U=16, d=25_557_032, E=4, M=3, gamma=0.9, iters=3, gammas=(0.5, 0.9, 0.99),
                     per_user_books=False),
    "cfg4": Workload("cfg4", 4, U=8, d=138_357_544, E=3, M=2, gamma=0.9, iters=3, beta=1.0, alpha=1e-3,
                     nseg=16, seg_alpha_range=(1e-5, 1e-2)),
    "cfg5": Workload("cfg5", 5, U=4, d=1_000_000_000, E=5, M=2, gamma=0.95, iters=2, beta=0.7,
                     alpha=1e-4, outlier_frac=1e-4, outlier_scale=100.0),
}


def gennorm_numpy(rng: np.random.Generator, n: int, beta: float, alpha: float) -> np.ndarray:
    g = rng.gamma(1.0 / beta, 1.0, size=n) ** (1.0 / beta)
    s = rng.integers(0, 2, size=n) * 2 - 1
    return (alpha * s * g).astype(np.float32)


def user_gradient_numpy(w: Workload, it: int, user: int) -> np.ndarray:
    """One user's flat gradient for one iteration (host, NumPy generator)."""
    rng = np.random.default_rng(seed_for(w.cfg, it, user))
    beta, alpha = w.user_params(user)
    x = gennorm_numpy(rng, w.d, beta, 1.0)
    sa = w.seg_alphas()
    if sa is None:
        x *= np.float32(alpha)
    else:
        off = 0
        for k, n in enumerate(w.seg_len):
            x[off:off + n] *= np.float32(sa[k])
            off += n
    if w.outlier_frac > 0:
        mask = rng.random(w.d) < w.outlier_frac
        x[mask] *= np.float32(w.outlier_scale)
    return x


def user_gradient_torch(w: Workload, it: int, user: int, device, out=None):
    """Same recipe drawn with torch's device generator (values differ from the NumPy draw;
    whichever array is drawn is handed to both the oracle and the GPU path)."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed_for(w.cfg, it, user))
    beta, alpha = w.user_params(user)
    if out is None:
        out = torch.empty(w.d, dtype=torch.float32, device=device)
    step = 1 << 26
    sa = w.seg_alphas()
    for o in range(0, w.d, step):
        n = min(step, w.d - o)
        conc = torch.full((n,), 1.0 / beta, dtype=torch.float32, device=device)
        gam = torch._standard_gamma(conc, generator=gen).pow_(1.0 / beta)
        sign = torch.randint(0, 2, (n,), generator=gen, device=device, dtype=torch.float32).mul_(2).sub_(1)
        gam.mul_(sign)
        if w.outlier_frac > 0:
            mask = torch.rand(n, generator=gen, device=device) < w.outlier_frac
            gam = torch.where(mask, gam * w.outlier_scale, gam)
        out[o:o + n] = gam
        del conc, gam, sign
    if sa is None:
        out.mul_(alpha)
    else:
        off = 0
        for k, n in enumerate(w.seg_len):
            out[off:off + n].mul_(float(sa[k]))
            off += n
    return out


def bias_for_max(max_abs: float, E: int) -> int:
    """The workloads' rule: the largest exponent of the format covers max|v|, i.e.
    (2^E - 2) - bias = floor(log2 max|v|)."""
    if not np.isfinite(max_abs) or max_abs <= 0:
        return (1 << (E - 1)) - 1
    return ((1 << E) - 2) - int(np.floor(np.log2(float(max_abs))))


def bias_table(v_abs_max_per_user_seg: np.ndarray, E: int) -> np.ndarray:
    """[U][nseg] biases from the per-(user, segment) max |g + gamma m|."""
    f = np.vectorize(lambda x: bias_for_max(x, E))
    return f(np.asarray(v_abs_max_per_user_seg, dtype=np.float64)).astype(np.int32)
