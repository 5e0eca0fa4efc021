"""CPU tests of the buffer-size tuner (Gaussian process + expected improvement, Sec. IV-B).
The search itself is stochastic ("parity unpinned"): only its parts with closed forms are
compared with numbers; the loop is checked by properties."""
from __future__ import annotations

import math

import numpy as np

from paper_2302_12445_amd.tuner import (MB, BufferSizeTuner, GaussianProcess, expected_improvement,
                                        grid_search, random_search)


def test_gp_interpolates_and_is_uncertain_away_from_data():
    x = np.array([0.0, 0.2, 0.45, 0.7, 1.0])
    y = np.sin(3 * x) + 0.5 * x
    gp = GaussianProcess(noise=1e-6)
    gp.fit(x, y)
    mu, sd = gp.predict(x)
    assert np.allclose(mu, y, atol=1e-3)
    assert np.all(sd < 0.02)
    mu2, sd2 = gp.predict(np.array([0.1, 0.575, 0.85]))
    assert np.all(sd2 > sd.max())
    assert np.allclose(mu2, np.sin(3 * np.array([0.1, 0.575, 0.85])) + 0.5 * np.array([0.1, 0.575, 0.85]), atol=0.15)


def test_expected_improvement_matches_sampling():
    rng = np.random.default_rng(0)
    for mu, sigma, best, xi in ((1.0, 0.5, 1.2, 0.1), (0.0, 1.0, 0.0, 0.0), (2.0, 0.3, 1.0, 0.1)):
        f = rng.normal(mu, sigma, size=2_000_000)
        mc = np.maximum(f - best - xi, 0.0).mean()
        ei = expected_improvement(np.array([mu]), np.array([sigma]), best, xi)[0]
        assert math.isclose(ei, mc, rel_tol=0.02, abs_tol=2e-3)
    # no uncertainty, no expected gain below the incumbent
    assert expected_improvement(np.array([0.0]), np.array([1e-9]), 1.0, 0.1)[0] < 1e-12


def _objective(noise, rng):
    # smooth, single peak at 35 MB, like the paper's buffer-size example for DenseNet-201
    def f(x_bytes):
        x = x_bytes / MB
        return 100.0 - 0.02 * (x - 35.0) ** 2 + (rng.normal(0, noise) if noise else 0.0)
    return f


def test_tuner_protocol():
    t = BufferSizeTuner()
    assert t.suggest() == 25 * MB                      # default start of the paper
    t.observe(25 * MB, 90.0)
    second = t.suggest()
    assert second == 100 * MB                          # far side of the range
    t.observe(second, 50.0)
    seen = {25 * MB, second}
    f = _objective(0.0, None)
    for _ in range(10):
        x = t.suggest()
        assert 1 * MB <= x <= 100 * MB and x not in seen
        seen.add(x)
        t.observe(x, f(x))
    bx, by = t.best()
    assert by == max(t.ys) and bx in seen


def test_tuner_finds_the_peak_in_few_trials_and_beats_random_search():
    wins, bo_scores, rnd_scores = 0, [], []
    for seed in range(10):
        rng = np.random.default_rng(100 + seed)
        f = _objective(0.05, rng)
        t = BufferSizeTuner(seed=seed)
        bx, by = t.run(f, 12)
        clean = _objective(0.0, None)
        bo_scores.append(clean(bx))
        rx, _, _ = random_search(f, 12, seed=seed)
        rnd_scores.append(clean(rx))
        wins += clean(bx) >= clean(rx)
        assert clean(bx) >= clean(25 * MB) - 0.2         # never worse than the default start
    assert np.mean(bo_scores) > 99.5                     # within 5 MB of the peak on average
    assert np.mean(bo_scores) >= np.mean(rnd_scores)
    assert wins >= 6


def test_grid_search_baseline():
    x, y, ys = grid_search(_objective(0.0, None), 12)
    assert len(ys) == 12 and y == max(ys) and abs(x / MB - 35) <= 5
