"""Whole runs: asynchronous Local-SGD with Delayed Nesterov + DyLU (Alg. 2 + Alg. 3 +
Eq. DyLU, workers running the inner loop of Alg. 1), and an independently written
synchronous DiLoCo loop (Alg. 1) used to pin the synchronous special case.
"""
from __future__ import annotations

import numpy as np

from . import lm
from .optim import (AdamW, AsyncBuffer, DelayedNesterov, delay_compensated, dylu_steps, nesterov_step,
                    poly_weight, pseudo_gradient)
from .scheduler import event_trace


class Worker:
    def __init__(self, idx, theta, cfg, stream, dtype):
        self.idx = idx
        self.theta = theta.copy()
        self.theta_start = theta.copy()
        self.opt = AdamW(theta.size, dtype, cfg["beta1"], cfg["beta2"], cfg["adam_eps"], cfg["wd"],
                         lm.n_decayed(cfg))
        self.stream = stream
        self.losses = []

    def restart(self, theta):
        self.theta = theta.copy()
        self.theta_start = theta.copy()

    def local_steps(self, n, cfg, lrs=None):
        """Inner loop of Alg. 1: n times (batch, loss, gradient, AdamW)."""
        toks = self.stream.take(n)
        for s in range(n):
            loss, grad = lm.loss_and_grad(self.theta, toks[s], cfg)
            self.opt.step(self.theta, grad, cfg["lr"] if lrs is None else lrs[s])
            self.losses.append(float(loss))


def run_async(cfg, theta0, make_stream, dtype=np.float32, n_events=None, log=None, rule=None):
    """Returns dict(theta, m, delta, t, losses[k][...], steps, groups, workers).

    rule (optional) selects one of the paper's comparison methods on top of the same loop:
      dict(kind="buffer")                         Async. Buffer with the configured N
      dict(poly_exponent=0.5)                     Async. DiLoCo + Poly
      dict(poly_exponent=0.5, staleness_threshold=10)   ... + PolyThres (stale updates dropped)
      dict(dc_lambda=lam)                         Async. DiLoCo + Delay Comp.
    Staleness of an update = server events applied since its worker (re)started."""
    theta0 = theta0.astype(dtype)
    k = cfg["k"]
    steps = dylu_steps(cfg["speeds"], cfg["H"])
    n_events = cfg["n_events"] if n_events is None else n_events
    groups = event_trace(cfg["speeds"], steps, cfg["tau_grace"], n_events)
    rule = rule or {}
    if rule.get("kind") == "buffer":
        server = AsyncBuffer(theta0, cfg["outer_lr"], cfg["outer_beta"], cfg["N"])
    else:
        server = DelayedNesterov(theta0, cfg["outer_lr"], cfg["outer_beta"], cfg["N"], cfg["dn_c"])
    workers = [Worker(i, theta0, cfg, make_stream(i), dtype) for i in range(k)]
    t_restart = [0] * k
    stale_log = []
    for w in workers:                       # train(W, theta) before the loop
        w.local_steps(int(steps[w.idx]), cfg)
    for g in groups:
        for (wi, _t) in g["events"]:
            w = workers[wi]
            stale = server.t - t_restart[wi]
            stale_log.append(stale)
            thr = rule.get("staleness_threshold", -1)
            if thr >= 0 and stale > thr:
                continue                         # PolyThres: the update is dropped
            pg = pseudo_gradient(w.theta_start, w.theta)
            if rule.get("dc_lambda", 0.0):
                pg = delay_compensated(pg, server.theta, w.theta_start, rule["dc_lambda"])
            if rule.get("poly_exponent", 0.0):
                pg = pg * dtype(poly_weight(stale, rule["poly_exponent"]))
            server.event(pg)
            if log is not None:
                log(server, wi)
        if g["complete"]:                   # train(W_completed, theta)
            for (wi, _t) in g["events"]:
                workers[wi].restart(server.theta)
                t_restart[wi] = server.t
            if g is not groups[-1]:
                for (wi, _t) in g["events"]:
                    workers[wi].local_steps(int(steps[wi]), cfg)
    return dict(theta=server.theta, m=server.m, delta=server.delta, t=server.t,
                losses=[w.losses for w in workers], steps=steps, groups=groups, workers=workers,
                staleness=stale_log)


def run_diloco_sync(cfg, theta0, make_stream, n_outer, H, dtype=np.float32):
    """Alg. 1 with AdamW inside and Nesterov (Eq. nesterov) outside, written on its own."""
    theta = theta0.astype(dtype).copy()
    m = np.zeros_like(theta)
    k = cfg["k"]
    opts = [AdamW(theta.size, dtype, cfg["beta1"], cfg["beta2"], cfg["adam_eps"], cfg["wd"],
                  lm.n_decayed(cfg)) for _ in range(k)]
    streams = [make_stream(i) for i in range(k)]
    losses = [[] for _ in range(k)]
    for _ in range(n_outer):
        deltas = []
        for i in range(k):
            th = theta.copy()
            toks = streams[i].take(H)
            for s in range(H):
                loss, grad = lm.loss_and_grad(th, toks[s], cfg)
                opts[i].step(th, grad, cfg["lr"])
                losses[i].append(float(loss))
            deltas.append(theta - th)
        mean_delta = sum(deltas) / dtype(k)
        theta, m = nesterov_step(theta, m, mean_delta, cfg["outer_lr"], cfg["outer_beta"])
    return dict(theta=theta, m=m, losses=losses)
