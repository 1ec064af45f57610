"""Inner and outer optimisers, the pseudo-gradient and DyLU.

AdamW is the paper's InnerOpt "with default values" and weight decay 0.1 (Optimization
Challenge section; hyper-parameter table); its state stays on the worker and is never reset
between rounds (appendix, Inner Optimizer States).  Reading of "default": beta1 0.9, beta2
0.999, eps 1e-8 added outside the square root, bias-corrected moments, decoupled decay
multiplied by the learning rate, decay on matrices and embeddings only.

The outer optimiser is Delayed Nesterov, taken step by step from Alg. 3; plain Nesterov is
Eq. (nesterov).  DyLU is Eq. (DyLU).
"""
from __future__ import annotations

import math
import numpy as np


class AdamW:
    """Per-worker persistent state (m, v, step count n)."""

    def __init__(self, P, dtype, beta1=0.9, beta2=0.999, eps=1e-8, wd=0.1, n_decayed=None):
        self.m = np.zeros(P, dtype=dtype)
        self.v = np.zeros(P, dtype=dtype)
        self.n = 0
        self.beta1, self.beta2, self.eps, self.wd = beta1, beta2, eps, wd
        self.n_decayed = P if n_decayed is None else n_decayed

    def step(self, theta, grad, lr):
        """In-place update of theta; returns theta."""
        t = theta.dtype.type
        self.n += 1
        b1, b2 = t(self.beta1), t(self.beta2)
        self.m[...] = b1 * self.m + (t(1.0) - b1) * grad
        self.v[...] = b2 * self.v + (t(1.0) - b2) * grad * grad
        mhat = self.m / t(1.0 - self.beta1 ** self.n)
        vhat = self.v / t(1.0 - self.beta2 ** self.n)
        upd = mhat / (np.sqrt(vhat) + t(self.eps))
        upd[:self.n_decayed] += t(self.wd) * theta[:self.n_decayed]
        theta -= t(lr) * upd
        return theta


def pseudo_gradient(theta_start, theta_worker):
    """delta_i = theta^(t-1) - theta_i^(t)  (Alg. 1, last line of the worker loop)."""
    return theta_start - theta_worker


def nesterov_step(theta, m, g, lr, beta):
    """Eq. (nesterov): returns (theta_next, m_next)."""
    t = theta.dtype.type
    m_next = t(beta) * m + g
    theta_next = theta - t(lr) * (t(beta * beta) * m + t(1.0 + beta) * g)
    return theta_next, m_next


class DelayedNesterov:
    """Server state (theta, m, Delta, t) and one sync() event per call -- Alg. 3."""

    def __init__(self, theta0, lr, beta, N, c=0.0):
        if not (0.0 <= c <= 1.0 / N + 1e-12):
            raise ValueError("momentum activation c must lie in [0, 1/N]")
        self.theta = theta0.copy()
        self.m = np.zeros_like(theta0)
        self.delta = np.zeros_like(theta0)
        self.t = 0
        self.lr, self.beta, self.N, self.c = lr, beta, int(N), c

    def event(self, g):
        f = self.theta.dtype.type
        N, c, beta, lr = self.N, self.c, self.beta, self.lr
        self.delta += g
        if (self.t + 1) % N == 0:
            self.m = f(beta) * self.m + self.delta / f(N)
            self.theta = self.theta - f(lr) * (f((1.0 - c * N + c) * beta) * self.m + g / f(N))
            self.delta = np.zeros_like(self.delta)
        else:
            self.theta = self.theta - f(lr) * (f(c * beta) * self.m + g / f(N))
        self.t += 1
        return self.theta


# ---- the comparison rules of the "Existing Fixes" paragraph (Optimization Challenge section) ----
def poly_weight(staleness, exponent=0.5):
    """Async. DiLoCo + Poly: g <- (1 + staleness)^-0.5 g."""
    return (1.0 + float(staleness)) ** (-exponent)


def delay_compensated(g, theta_now, theta_then, lam):
    """Async. DiLoCo + Delay Comp.: first-order correction of a stale pseudo-gradient with the
    diagonal outer-product approximation of the Hessian, g + lam * g*g*(theta_now - theta_then)."""
    t = g.dtype.type
    return g + t(lam) * g * g * (theta_now - theta_then)


class AsyncBuffer:
    """Async. Buffer: pseudo-gradients are accumulated first-in first-out; every N-th one the
    average is applied with one Nesterov step (Eq. nesterov); parameters do not move in between."""

    def __init__(self, theta0, lr, beta, N):
        self.theta = theta0.copy()
        self.m = np.zeros_like(theta0)
        self.delta = np.zeros_like(theta0)
        self.t = 0
        self.lr, self.beta, self.N = lr, beta, int(N)

    def event(self, g):
        f = self.theta.dtype.type
        self.delta += g
        if (self.t + 1) % self.N == 0:
            gbar = self.delta / f(self.N)
            self.m = f(self.beta) * self.m + gbar
            self.theta = self.theta - f(self.lr) * (f(self.beta) * self.m + gbar)
            self.delta = np.zeros_like(self.delta)
        self.t += 1
        return self.theta


def dylu_steps(speeds, H):
    """Eq. (DyLU): floor(v_i / max v * H), evaluated in fp64 in that order; a result of 0
    is raised to 1 (a zero-step job would return a zero pseudo-gradient in zero time)."""
    v = np.asarray(speeds, dtype=np.float64)
    if v.ndim != 1 or v.size == 0 or not np.all(np.isfinite(v)) or np.any(v <= 0) or H < 1:
        raise ValueError("speeds must be finite and positive, H >= 1")
    vmax = float(np.max(v))
    return np.array([max(1, int(math.floor((float(x) / vmax) * float(H)))) for x in v],
                    dtype=np.int32)
