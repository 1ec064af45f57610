"""Pins for the oracle's whole-run loops (CPU only)."""
import numpy as np
import pytest

import als_inputs as I
from oracle import lm, run
from oracle.optim import AdamW

SMALL = dict(I._COMMON, L=1, d=16, h=2, ff=32, V=19, S=5, B=2, dtype="f32", k=3,
             speeds=np.array([2.0, 2.0, 2.0]), H=3, N=3, n_events=6)


def _stream(cfg):
    return lambda i: I.TokenStream(cfg["seed"], i, cfg["B"], cfg["S"], cfg["V"])


def test_sync_special_case_equals_diloco():
    # equal speeds, equal H, tau_grace = 0, N = k, c = 0: the asynchronous loop with Delayed
    # Nesterov must reproduce Alg. 1 with Nesterov on the averaged pseudo-gradient.
    cfg = dict(SMALL)
    th0 = I.theta0(lm.param_layout(cfg), 0).astype(np.float64)
    a = run.run_async(cfg, th0, _stream(cfg), dtype=np.float64)
    s = run.run_diloco_sync(cfg, th0, _stream(cfg), n_outer=2, H=3, dtype=np.float64)
    assert [len(g["events"]) for g in a["groups"]] == [3, 3]
    np.testing.assert_allclose(a["theta"], s["theta"], rtol=0, atol=1e-12)
    np.testing.assert_allclose(a["m"], s["m"], rtol=0, atol=1e-12)
    for la, ls in zip(a["losses"], s["losses"]):
        np.testing.assert_allclose(la, ls[:len(la)], rtol=1e-12)
    assert np.abs(a["theta"] - th0).max() > 1e-3        # something was learned


def test_adamw_state_persists_across_rounds():
    cfg = dict(SMALL, k=1, speeds=np.array([1.0]), N=1, n_events=2, H=2)
    th0 = I.theta0(lm.param_layout(cfg), 0).astype(np.float64)
    r = run.run_async(cfg, th0, _stream(cfg), dtype=np.float64, n_events=2)
    w = r["workers"][0]
    # two rounds of 2 steps were trained (the third restart trains nothing)
    assert w.opt.n == 4 and len(w.losses) == 4
    # replay by hand: round 2 starts from the server model but keeps m, v and the step count
    st = I.TokenStream(cfg["seed"], 0, cfg["B"], cfg["S"], cfg["V"])
    opt = AdamW(th0.size, np.float64, n_decayed=lm.n_decayed(cfg))
    th = th0.copy()
    for tok in st.take(2):
        opt.step(th, lm.loss_and_grad(th, tok, cfg)[1], cfg["lr"])
    g = th0 - th
    theta1 = th0 - 0.7 * (0.9 * g + g)          # N = 1: Nesterov from m = 0
    th = theta1.copy()
    losses = []
    for tok in st.take(2):
        l, gr = lm.loss_and_grad(th, tok, cfg)
        losses.append(float(l))
        opt.step(th, gr, cfg["lr"])
    np.testing.assert_allclose(w.losses[2:], losses, rtol=1e-12)
    assert opt.n == 4


def test_tiny_run_lowers_loss_and_follows_trace():
    cfg = I.workload("tiny")
    th0 = I.theta0(lm.param_layout(cfg), 0)
    seen = []
    r = run.run_async(cfg, th0, _stream(cfg), log=lambda srv, wi: seen.append((srv.t, wi)))
    assert [w for _, w in seen] == [0, 1, 2, 3, 0, 1, 0, 2, 3, 0, 1, 2]
    assert r["t"] == 12 and r["theta"].dtype == np.float32
    assert r["steps"].tolist() == [1, 2, 3, 5]
    assert np.mean(r["losses"][3][-3:]) < np.mean(r["losses"][3][:3]) - 0.1


def test_staleness_counts_and_threshold_drop():
    # speeds (1, 1.5, 2, 3), H = 5: hand-traced order 0 1 2 3 0 1 (0 2) 3 (0 1) 2; staleness of
    # an update = server events since its worker restarted: first four 0 1 2 3, then w0 (restarted
    # after event 1, synced as event 5) 3, w1 3, w0 1, w2 4 ...
    cfg = dict(I.workload("tiny"), N=1)
    th0 = I.theta0(lm.param_layout(cfg), 0)
    r = run.run_async(cfg, th0, _stream(cfg), n_events=8, rule=dict(poly_exponent=0.5))
    assert r["staleness"] == [0, 1, 2, 3, 3, 3, 1, 4]
    # with a threshold of 2 every update staler than 2 is dropped and does not count as an event,
    # so later updates look less stale: 0 1 2 [3 dropped] then w0: 3 - 1 = 2, w1: 4 - 2 = 2,
    # w0: 5 - 4 = 1, w2: 6 - 3 = 3 [dropped]
    r2 = run.run_async(cfg, th0, _stream(cfg), n_events=8, rule=dict(poly_exponent=0.5, staleness_threshold=2))
    assert r2["staleness"] == [0, 1, 2, 3, 2, 2, 1, 3]
    assert r2["t"] == 6
