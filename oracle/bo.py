"""Bayesian-optimisation autotuner of the trigger thresholds (checker): TEST INFRASTRUCTURE.

Sec. 3.3 ("BO autotuner") and the appendix "Design and Performance Evaluation of BO": the thresholds
(R1, R2) in (0,1)^2 are tuned by Bayesian optimisation of the measured time per accepted token (TPT,
to be minimised): Gaussian-process regression with a Matern kernel as the surrogate, Expected
Improvement with exploration parameter 0.1 as the acquisition function, one random initial sample,
16 samples in all.  Written out plainly in numpy fp64: build the kernel matrix, solve, evaluate.

Readings (the paper names the ingredients and no more):
* Matern smoothness nu = 5/2: k(r) = (1 + sqrt5 r/l + 5 r^2 / (3 l^2)) exp(-sqrt5 r/l), r the
  Euclidean distance in the (R1, R2) plane, unit signal variance on standardised observations;
* the observations are standardised (zero mean, unit population standard deviation; a constant set
  keeps scale 1) before regression and the posterior is mapped back;
* fixed hyper-parameters passed in by the caller (length scale l, observation noise variance added
  to the diagonal): no marginal-likelihood fit, so that the suggestion is a pure function of its inputs;
* EI for MINIMISATION on the standardised scale: with I = y_best - mu - xi and s the posterior
  standard deviation, EI = I Phi(I/s) + s phi(I/s), and EI = max(I, 0) where s = 0;
* the next sample is the maximiser of EI over the midpoints of a uniform g x g grid of (0,1)^2
  (lowest index among equal values, R1 varying slowest), not a continuous search;
* the random initial sample is an input (drawn by the caller).
"""
from __future__ import annotations

import math
from typing import Sequence, Tuple

import numpy as np


def matern52(a: np.ndarray, b: np.ndarray, length_scale: float) -> np.ndarray:
    """Kernel matrix between point sets a [n][2] and b [m][2]."""
    a = np.asarray(a, dtype=np.float64).reshape(-1, 2)
    b = np.asarray(b, dtype=np.float64).reshape(-1, 2)
    r = np.sqrt(((a[:, None, :] - b[None, :, :]) ** 2).sum(-1)) / float(length_scale)
    s5 = math.sqrt(5.0)
    return (1.0 + s5 * r + (5.0 / 3.0) * r * r) * np.exp(-s5 * r)


def standardise(y: np.ndarray) -> Tuple[np.ndarray, float, float]:
    y = np.asarray(y, dtype=np.float64)
    mean = float(y.mean())
    scale = float(y.std())
    if not scale > 0.0:
        scale = 1.0
    return (y - mean) / scale, mean, scale


def posterior(x, y, length_scale: float, noise: float, q) -> Tuple[np.ndarray, np.ndarray]:
    """GP posterior mean and standard deviation at the query points q [m][2], in the units of y."""
    x = np.asarray(x, dtype=np.float64).reshape(-1, 2)
    q = np.asarray(q, dtype=np.float64).reshape(-1, 2)
    ys, mean, scale = standardise(y)
    K = matern52(x, x, length_scale) + float(noise) * np.eye(len(x))
    Ks = matern52(x, q, length_scale)            # [n][m]
    alpha = np.linalg.solve(K, ys)
    mu = Ks.T @ alpha
    v = np.linalg.solve(K, Ks)
    var = 1.0 - np.einsum("nm,nm->m", Ks, v)     # k(q, q) = 1
    sd = np.sqrt(np.maximum(var, 0.0))
    return mean + scale * mu, scale * sd


def _phi(z):
    return np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)


def _Phi(z):
    return np.array([0.5 * (1.0 + math.erf(float(v) / math.sqrt(2.0))) for v in np.ravel(z)], dtype=np.float64).reshape(np.shape(z))


def expected_improvement(mu_s: np.ndarray, sd_s: np.ndarray, best_s: float, xi: float) -> np.ndarray:
    """EI for minimisation on the standardised scale."""
    imp = best_s - mu_s - xi
    out = np.maximum(imp, 0.0)
    pos = sd_s > 0.0
    z = imp[pos] / sd_s[pos]
    out[pos] = imp[pos] * _Phi(z) + sd_s[pos] * _phi(z)
    return out


def grid_points(g: int) -> np.ndarray:
    """Midpoints of a uniform g x g grid of (0,1)^2, R1 varying slowest."""
    c = (np.arange(g, dtype=np.float64) + 0.5) / g
    return np.stack(np.meshgrid(c, c, indexing="ij"), -1).reshape(-1, 2)


def suggest(x, y, length_scale: float, noise: float, xi: float, g: int) -> Tuple[Tuple[float, float], float]:
    """Next (R1, R2) to try and its EI (standardised units)."""
    x = np.asarray(x, dtype=np.float64).reshape(-1, 2)
    ys, _, _ = standardise(y)
    q = grid_points(g)
    K = matern52(x, x, length_scale) + float(noise) * np.eye(len(x))
    Ks = matern52(x, q, length_scale)
    mu = Ks.T @ np.linalg.solve(K, ys)
    var = 1.0 - np.einsum("nm,nm->m", Ks, np.linalg.solve(K, Ks))
    sd = np.sqrt(np.maximum(var, 0.0))
    ei = expected_improvement(mu, sd, float(ys.min()), xi)
    i = int(np.argmax(ei))
    return (float(q[i, 0]), float(q[i, 1])), float(ei[i])


def tune(objective, first: Sequence[float], n_samples: int, length_scale: float, noise: float, xi: float, g: int):
    """The autotuner's loop: `first` is the random initial sample; every further sample is the
    suggestion for what has been observed so far.  Returns (samples, values, index of the best)."""
    xs = [tuple(float(v) for v in first)]
    ys = [float(objective(*xs[0]))]
    while len(xs) < n_samples:
        nxt, _ = suggest(xs, ys, length_scale, noise, xi, g)
        xs.append(nxt)
        ys.append(float(objective(*nxt)))
    return xs, ys, int(np.argmin(ys))
