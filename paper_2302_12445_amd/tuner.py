"""Run-time tuning of the fusion buffer size x by Bayesian optimisation.

Paper Section IV-B: the throughput P(x) of the running system is an unknown function of
the buffer size x; it is measured for a default x1 = 25 MB over a few steps, a Gaussian
process is fitted to the observations (x_i, P(x_i)), and the next x maximises the
expected improvement (EI) over the best observation; the EI exploration parameter is 0.1
and x ranges over about 1 MB .. 100 MB; tens of trials suffice.  Random and grid search
are the baselines the paper compares against (Section VI-G).

Host-side numpy only; the objective is whatever the caller measures (here: iterations
per second of the two-stream schedule on the GPU).  The search is stochastic where it
breaks ties, so its result is checked by property ("not worse than the default"), not
against stored values.
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

MB = 1 << 20


def _matern52(a: np.ndarray, b: np.ndarray, length: float) -> np.ndarray:
    d = np.abs(a[:, None] - b[None, :]) / length
    s = math.sqrt(5.0) * d
    return (1.0 + s + s * s / 3.0) * np.exp(-s)


class GaussianProcess:
    """Zero-mean GP with a Matern-5/2 kernel on inputs scaled to [0, 1] and targets
    standardised; the length scale is chosen among a few values by marginal likelihood."""

    LENGTHS = (0.05, 0.1, 0.2, 0.4, 0.8)

    def __init__(self, noise: float = 1e-3):
        self.noise = noise
        self.x: Optional[np.ndarray] = None

    def fit(self, x: Sequence[float], y: Sequence[float]) -> None:
        self.x = np.asarray(x, float)
        y = np.asarray(y, float)
        self.y_mean = float(y.mean())
        self.y_std = float(y.std()) or 1.0
        t = (y - self.y_mean) / self.y_std
        best = None
        for length in self.LENGTHS:
            K = _matern52(self.x, self.x, length) + self.noise * np.eye(len(t))
            Lc = np.linalg.cholesky(K)
            alpha = np.linalg.solve(Lc.T, np.linalg.solve(Lc, t))
            loglik = -0.5 * float(t @ alpha) - float(np.log(np.diag(Lc)).sum())
            if best is None or loglik > best[0]:
                best = (loglik, length, Lc, alpha)
        _, self.length, self.Lc, self.alpha = best

    def predict(self, xq: Sequence[float]) -> Tuple[np.ndarray, np.ndarray]:
        xq = np.asarray(xq, float)
        Ks = _matern52(xq, self.x, self.length)
        mu = Ks @ self.alpha
        v = np.linalg.solve(self.Lc, Ks.T)
        var = np.maximum(1.0 + self.noise - np.sum(v * v, axis=0), 1e-12)
        return mu * self.y_std + self.y_mean, np.sqrt(var) * self.y_std


def expected_improvement(mu: np.ndarray, sigma: np.ndarray, best: float, xi: float) -> np.ndarray:
    """EI for maximisation: E[max(f - best - xi, 0)] under N(mu, sigma^2)."""
    imp = mu - best - xi
    z = imp / sigma
    cdf = 0.5 * (1.0 + np.vectorize(math.erf)(z / math.sqrt(2.0)))
    pdf = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
    return imp * cdf + sigma * pdf


class BufferSizeTuner:
    """suggest() / observe() loop over the buffer size in bytes."""

    def __init__(self, lo_bytes: int = 1 * MB, hi_bytes: int = 100 * MB, first_bytes: int = 25 * MB,
                 xi: float = 0.1, grid: int = 397, seed: int = 0):
        self.lo, self.hi, self.first, self.xi = lo_bytes, hi_bytes, first_bytes, xi
        self.cand = np.linspace(0.0, 1.0, grid)
        self.rng = np.random.default_rng(seed)
        self.xs: List[float] = []   # scaled to [0, 1]
        self.ys: List[float] = []
        self.gp = GaussianProcess()

    def _scale(self, b: float) -> float:
        return (b - self.lo) / (self.hi - self.lo)

    def _bytes(self, u: float) -> int:
        return int(round(self.lo + u * (self.hi - self.lo)))

    def suggest(self) -> int:
        if not self.xs:
            return int(self.first)
        if len(self.xs) == 1:  # one point says nothing about the slope: probe the far side
            return self._bytes(0.0 if self.xs[0] > 0.5 else 1.0)
        self.gp.fit(self.xs, self.ys)
        mu, sigma = self.gp.predict(self.cand)
        # xi is relative to the spread of the observations, as the targets are standardised
        ei = expected_improvement(mu, sigma, max(self.ys), self.xi * self.gp.y_std)
        seen = np.min(np.abs(self.cand[:, None] - np.asarray(self.xs)[None, :]), axis=1) < 0.5 / len(self.cand)
        ei[seen] = -np.inf
        top = np.flatnonzero(ei >= ei.max() - 1e-15)
        return self._bytes(float(self.cand[self.rng.choice(top)]))

    def observe(self, x_bytes: int, throughput: float) -> None:
        self.xs.append(self._scale(float(x_bytes)))
        self.ys.append(float(throughput))

    def best(self) -> Tuple[int, float]:
        i = int(np.argmax(self.ys))
        return self._bytes(self.xs[i]), self.ys[i]

    def run(self, measure: Callable[[int], float], trials: int) -> Tuple[int, float]:
        for _ in range(trials):
            x = self.suggest()
            self.observe(x, measure(x))
        return self.best()


def random_search(measure: Callable[[int], float], trials: int, lo_bytes: int = 1 * MB,
                  hi_bytes: int = 100 * MB, first_bytes: int = 25 * MB, seed: int = 0) -> Tuple[int, float, List[float]]:
    rng = np.random.default_rng(seed)
    xs = [first_bytes] + [int(rng.uniform(lo_bytes, hi_bytes)) for _ in range(trials - 1)]
    ys = [measure(x) for x in xs]
    i = int(np.argmax(ys))
    return xs[i], ys[i], ys


def grid_search(measure: Callable[[int], float], trials: int, lo_bytes: int = 1 * MB,
                hi_bytes: int = 100 * MB) -> Tuple[int, float, List[float]]:
    xs = [int(v) for v in np.linspace(lo_bytes, hi_bytes, trials)]
    ys = [measure(x) for x in xs]
    i = int(np.argmax(ys))
    return xs[i], ys[i], ys
