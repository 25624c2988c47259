"""Seeded synthetic inputs for the constrained layer-wise compression problem (Eq. 1, Sec. 3.1).

This module only *draws inputs*: an integer timing table ``tau[L, S]``, K error tables
``err[K, L, S]`` and a budget ``B``.  It contains none of the solver's arithmetic and is the one
piece of code that both the CPU oracle's tests and the GPU path's tests/benchmark use.

Shapes follow the workloads the paper describes: about 52-54 prunable layers and about 40
geometrically spaced sparsity levels for a ResNet-50 (Sec. 3.2, Sec. 4 "Setup"), B = 10^4 time
buckets (Sec. 4 "Setup"), 12 x 6 linear projections for BERT-base with the feed-forward layers
dominating the runtime (App. profile visualisations), errors that grow quadratically in the level
with a per-layer sensitivity drawn uniformly from (0, 1) (Eq. 4, Alg. 4).  The real timing tables
were measured on an inference engine and are not available; these tables stand in for them.

Recipe (all math in float64, one cast at the end, NumPy ``PCG64(seed)``; draw order: the L dense
times first, then the sensitivities ``c[k, l]`` row-major):

    p_s        = 1 - q**s                         s = 0 .. S-1   (s = 0 is the dense level)
    f_s        = 0.2 + 0.8 * (1 - p_s)**1.5       time factor, f_0 = 1
    scale      = X * B / sum_l d_l                X = speed-up target, so sum_l tau[l, 0] ~ X * B
    tau[l, s]  = int32(floor(d_l * f_s * scale + 0.5))
    err[k,l,s] = float32(c[k, l] * p_s**2)        err[k, l, 0] = +0.0
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    K: int
    L: int
    S: int
    B: int
    q: float          # kept fraction per level step: p_s = 1 - q**s
    speedup: float    # X
    dense: str        # how the dense layer times d_l are drawn
    sigma: float      # log-normal sigma of d_l (jitter sigma for "bert")
    grid: str = "geometric"   # "geometric": p_s = 1 - q**s;  "paper": the Sec. 4 "Setup" grid

    @property
    def cell_updates(self) -> int:
        """Nominal work K*L*S*B of the dynamic program (Sec. 3.2: O(|S| L T))."""
        return self.K * self.L * self.S * self.B


CONFIGS = {
    "tiny": Config("tiny", K=1, L=8, S=8, B=256, q=0.8, speedup=2.0, dense="lognormal", sigma=0.5),
    "rn50_k1": Config("rn50_k1", K=1, L=54, S=40, B=10000, q=0.9, speedup=2.5,
                      dense="lognormal", sigma=0.8),
    "rn50_k1024": Config("rn50_k1024", K=1024, L=54, S=40, B=10000, q=0.9, speedup=2.5,
                         dense="lognormal", sigma=0.8),
    "bert_k4096": Config("bert_k4096", K=4096, L=72, S=40, B=16384, q=0.9, speedup=3.0,
                         dense="bert", sigma=0.1),
    "stress_k256": Config("stress_k256", K=256, L=200, S=64, B=65536, q=0.93, speedup=4.0,
                          dense="lognormal", sigma=1.0),
    # the sizes Sec. 3.2 quotes for a ResNet-50 (L = 52, |S| = 42, T = 10^4) with the sparsity
    # grid of Sec. 4 "Setup", the error model of Eq. 4 and non-monotone timings (Sec. 3.1)
    "paper_rn50_k1024": Config("paper_rn50_k1024", K=1024, L=52, S=42, B=10000, q=0.0,
                               speedup=2.5, dense="lognormal", sigma=0.8, grid="paper"),
    # another additive constraint (Sec. 3.1: the same problem with parameters or FLOPs in place of
    # time): tau = remaining parameters of a ResNet-50's 53 convolutions and its classifier,
    # budget = 1 / speedup of the dense parameter count
    "rn50_params_k1024": Config("rn50_params_k1024", K=1024, L=54, S=40, B=10000, q=0.9,
                                speedup=4.0, dense="rn50_params", sigma=0.0),
    # Not benchmark lines: tables that take the other launches of the fill, for profiling them.
    # The stress recipe with looser speed-up targets leaves longer reduced rows: X = 3.8 about
    # 15.5 K reduced buckets and X = 3.0 about 26 K (one row in LDS updated in place by a
    # workgroup of twice the waves; the level record takes two rows in LDS or global rows there),
    # X = 2.5 about 32.6 K (rows in global memory, one workgroup per compute unit); the ResNet-50
    # recipe with ten times the buckets (global rows, two workgroups per compute unit); and the
    # ResNet-50 recipe with 128 levels (the instantiations for S > 64).
    "stress_x38_k256": Config("stress_x38_k256", K=256, L=200, S=64, B=65536, q=0.93,
                              speedup=3.8, dense="lognormal", sigma=1.0),
    "stress_x30_k256": Config("stress_x30_k256", K=256, L=200, S=64, B=65536, q=0.93,
                              speedup=3.0, dense="lognormal", sigma=1.0),
    "stress_x25_k256": Config("stress_x25_k256", K=256, L=200, S=64, B=65536, q=0.93,
                              speedup=2.5, dense="lognormal", sigma=1.0),
    "rn50_b100k_k1024": Config("rn50_b100k_k1024", K=1024, L=54, S=40, B=100000, q=0.9,
                               speedup=2.5, dense="lognormal", sigma=0.8),
    "rn50_s128_k1024": Config("rn50_s128_k1024", K=1024, L=54, S=128, B=10000, q=0.97,
                              speedup=2.5, dense="lognormal", sigma=0.8),
}


def resnet50_parameter_counts() -> np.ndarray:
    """Weights of the 53 convolutions and the classifier of the standard ResNet-50 architecture
    (7x7 stem, bottleneck stages of 3, 4, 6, 3 blocks with widths 64, 128, 256, 512 and a
    1x1 projection in the first block of each stage, 2048 x 1000 classifier), in network order."""
    counts = [7 * 7 * 3 * 64]
    inplanes = 64
    for width, blocks in ((64, 3), (128, 4), (256, 6), (512, 3)):
        for b in range(blocks):
            counts += [inplanes * width, 3 * 3 * width * width, width * 4 * width]
            if b == 0:
                counts.append(inplanes * 4 * width)
            inplanes = 4 * width
    counts.append(2048 * 1000)
    return np.asarray(counts, dtype=np.float64)


def level_grid(S: int, q: float) -> np.ndarray:
    """Sparsity of level s: p_s = 1 - q**s (float64)."""
    return 1.0 - np.power(q, np.arange(S, dtype=np.float64))


def paper_grid() -> np.ndarray:
    """Sec. 4 "Setup": S = {0} u {1 - (1 - 0.4) d^i, i = 0..40}, d = ((1-0.99)/(1-0.4))^(1/40)."""
    d = ((1.0 - 0.99) / (1.0 - 0.4)) ** (1.0 / 40.0)
    return np.concatenate([[0.0], 1.0 - 0.6 * np.power(d, np.arange(41, dtype=np.float64))])


def _generate_paper_shape(cfg: Config, rng, K: int):
    """Paper-shaped tables: the Sec. 4 grid (dense + 41 levels from 40 % to 99 % sparsity); sparse
    execution only pays off from about 40 % sparsity (time factor 0.1 + 1.35 (1-p)^0.9, 0.95 at
    p = 0.4) and every (layer, level) time carries 5 % log-normal measurement noise, so times are
    not monotone in the level (Sec. 3.1); errors follow Eq. 4: c_l (i / (|S| - 1))^2."""
    p = paper_grid()
    assert cfg.S == p.size
    d = rng.lognormal(0.0, cfg.sigma, size=cfg.L)
    f = np.where(p > 0, 0.1 + 1.35 * np.power(1.0 - p, 0.9), 1.0)
    noise = rng.lognormal(0.0, 0.05, size=(cfg.L, cfg.S))
    scale = cfg.speedup * cfg.B / d.sum()
    tau = np.floor(d[:, None] * f[None, :] * noise * scale + 0.5).astype(np.int32)
    c = rng.random((K, cfg.L))
    w = np.square(np.arange(cfg.S, dtype=np.float64) / (cfg.S - 1))
    err = (c[:, :, None] * w[None, None, :]).astype(np.float32)
    return np.ascontiguousarray(tau), np.ascontiguousarray(err), cfg.B


def generate(cfg: Config, seed: int = 0, K: int | None = None):
    """Return ``(tau int32[L,S], err float32[K,L,S], B)`` for ``cfg``.

    ``K`` overrides the number of candidates; because sensitivities are drawn row-major after the
    dense times, the first K' candidates of a larger draw equal a draw with K = K'.
    """
    K = cfg.K if K is None else int(K)
    rng = np.random.Generator(np.random.PCG64(seed))
    if cfg.grid == "paper":
        return _generate_paper_shape(cfg, rng, K)
    if cfg.dense == "lognormal":
        d = rng.lognormal(0.0, cfg.sigma, size=cfg.L)
    elif cfg.dense == "bert":
        base = np.array([1.0, 1.0, 1.0, 1.0, 4.0, 4.0])[np.arange(cfg.L) % 6]
        d = base * rng.lognormal(0.0, cfg.sigma, size=cfg.L)
    elif cfg.dense == "rn50_params":
        d = resnet50_parameter_counts()
        assert d.size == cfg.L
    else:
        raise ValueError(cfg.dense)
    p = level_grid(cfg.S, cfg.q)
    # time falls off slower than the kept fraction; a parameter count is exactly proportional
    f = (1.0 - p) if cfg.dense == "rn50_params" else 0.2 + 0.8 * np.power(1.0 - p, 1.5)
    scale = cfg.speedup * cfg.B / d.sum()
    tau = np.floor(d[:, None] * f[None, :] * scale + 0.5).astype(np.int32)
    c = rng.random((K, cfg.L))
    while True:
        zero = c == 0.0
        if not zero.any():
            break
        c[zero] = rng.random(int(zero.sum()))
    err = (c[:, :, None] * (p * p)[None, None, :]).astype(np.float32)
    return np.ascontiguousarray(tau), np.ascontiguousarray(err), cfg.B


def random_instance(rng: np.random.Generator, K: int, L: int, S: int, B: int, *,
                    tau_max: int | None = None, integer_err: int | None = None,
                    zero_tau_frac: float = 0.0, over_budget_frac: float = 0.0,
                    inf_err_frac: float = 0.0, layer_floor: int = 0, huge_tau_frac: float = 0.0,
                    err_scale: float = 1.0):
    """Unstructured random tables for tests (no monotonicity in s, Sec. 3.1: timings are
    non-linear and a sparse layer can be slower than the dense one).

    ``integer_err=m`` draws errors from {0..m-1} (sums exact in fp32, ties frequent); otherwise
    errors are uniform in [0, 1).  Fractions select entries forced to tau = 0, tau > B, err = +inf.
    ``layer_floor > 0`` adds a random per-layer offset in [0, layer_floor] to every time of the
    layer, so that the smallest time of a layer is well above zero.  ``huge_tau_frac`` forces
    entries to the largest int32; ``err_scale`` multiplies every error (a power of two far below
    one moves the errors into the fp32 subnormal range).
    """
    tau_max = max(1, B // 2) if tau_max is None else tau_max
    tau = rng.integers(0, tau_max + 1, size=(L, S), dtype=np.int64)
    if layer_floor > 0:
        tau += rng.integers(0, layer_floor + 1, size=(L, 1), dtype=np.int64)
    if zero_tau_frac > 0:
        tau[rng.random((L, S)) < zero_tau_frac] = 0
    if over_budget_frac > 0:
        m = rng.random((L, S)) < over_budget_frac
        tau[m] = B + 1 + rng.integers(0, 5, size=int(m.sum()))
    if huge_tau_frac > 0:
        tau[rng.random((L, S)) < huge_tau_frac] = 2 ** 31 - 1
    if integer_err is not None:
        err = rng.integers(0, integer_err, size=(K, L, S)).astype(np.float32)
    else:
        err = rng.random((K, L, S), dtype=np.float32)
    if err_scale != 1.0:
        err = (err * np.float32(err_scale)).astype(np.float32)
    if inf_err_frac > 0:
        err[rng.random((K, L, S)) < inf_err_frac] = np.inf
    return np.ascontiguousarray(tau.astype(np.int32)), np.ascontiguousarray(err), B
