"""Pins for the oracle's optimisers, DyLU and the scheduler (CPU only)."""
import math

import numpy as np
import pytest
import torch

from oracle.optim import AdamW, DelayedNesterov, dylu_steps, nesterov_step, pseudo_gradient
from oracle.scheduler import event_trace, flat_events


# ----------------------------------------------------------------------------- Nesterov
def test_nesterov_hand_worked_scalar(golden):
    G = golden("nesterov_scalar.txt")
    th, m = np.zeros(1), np.zeros(1)
    for k in range(4):
        th, m = nesterov_step(th, m, np.ones(1), 0.7, 0.9)
        assert th[0] == pytest.approx(G["nesterov_theta"][k], abs=1e-12)
        assert m[0] == pytest.approx(G["nesterov_m"][k], abs=1e-12)


def test_nesterov_matches_library_sgd_nesterov():
    rng = np.random.default_rng(3)
    th0 = rng.standard_normal(7)
    p = torch.nn.Parameter(torch.tensor(th0.copy()))
    opt = torch.optim.SGD([p], lr=0.7, momentum=0.9, dampening=0.0, nesterov=True)
    th, m = th0.copy(), np.zeros(7)
    for _ in range(6):
        g = rng.standard_normal(7)
        p.grad = torch.tensor(g.copy())
        opt.step()
        th, m = nesterov_step(th, m, g, 0.7, 0.9)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=0, atol=1e-13)


def test_sequential_application_identity_printed_in_paper(golden):
    G = golden("nesterov_scalar.txt")
    beta, eps = 0.9, 0.7
    rng = np.random.default_rng(0)
    g, m0, th0 = rng.standard_normal(5), rng.standard_normal(5), rng.standard_normal(5)
    th, m = th0.copy(), m0.copy()
    for _ in range(4):
        th, m = nesterov_step(th, m, g, eps, beta)
    np.testing.assert_allclose(m, G["seq4_coef_m_m"][0] * m0 + G["seq4_coef_m_g"][0] * g, atol=1e-12)
    np.testing.assert_allclose(
        th, th0 - eps * (G["seq4_coef_theta_g"][0] * g + G["seq4_coef_theta_m"][0] * m0), atol=1e-12)
    # the coefficients themselves, from the printed polynomials
    b = beta
    assert G["seq4_coef_theta_g"][0] == pytest.approx(4 + 4 * b + 3 * b**2 + 2 * b**3 + b**4, abs=1e-12)
    assert G["seq4_coef_theta_m"][0] == pytest.approx(b**2 * (1 + b + b**2 + b**3), abs=1e-12)


# ------------------------------------------------------------------------ Delayed Nesterov
@pytest.mark.parametrize("key,c,gkey", [("ones", 0.0, None), ("vary_c0", 0.0, "vary_g"),
                                        ("vary_c01", 0.1, "vary_g")])
def test_dn_hand_worked_scalar(golden, key, c, gkey):
    G = golden("dn_scalar.txt")
    gs = G[gkey] if gkey else [1.0] * 8
    dn = DelayedNesterov(np.zeros(1), 0.7, 0.9, 4, c)
    for e in range(8):
        dn.event(np.array([gs[e]]))
        assert dn.theta[0] == pytest.approx(G[key + "_theta"][e], abs=1e-12), e
        assert dn.m[0] == pytest.approx(G[key + "_m"][e], abs=1e-12), e
    assert dn.t == 8 and dn.delta[0] == 0.0


@pytest.mark.parametrize("c", [0.0, 0.3, 1.0])
def test_dn_with_buffer_one_is_nesterov(c):
    rng = np.random.default_rng(1)
    th0 = rng.standard_normal(11)
    dn = DelayedNesterov(th0, 0.7, 0.9, 1, c)
    th, m = th0.copy(), np.zeros(11)
    for _ in range(5):
        g = rng.standard_normal(11)
        dn.event(g)
        th, m = nesterov_step(th, m, g, 0.7, 0.9)
        np.testing.assert_allclose(dn.theta, th, atol=1e-13)
        np.testing.assert_allclose(dn.m, m, atol=1e-13)


def test_dn_period_equals_nesterov_on_mean_pseudogradient():
    rng = np.random.default_rng(2)
    N = 4
    th0 = rng.standard_normal(9)
    dn = DelayedNesterov(th0, 0.7, 0.9, N, 0.0)
    th, m = th0.copy(), np.zeros(9)
    for _ in range(3):
        gs = [rng.standard_normal(9) for _ in range(N)]
        for j, g in enumerate(gs):
            m_before = dn.m.copy()
            dn.event(g)
            if j < N - 1:       # momentum is delayed, buffer holds the running sum
                np.testing.assert_array_equal(dn.m, m_before)
                np.testing.assert_allclose(dn.delta, sum(gs[:j + 1]), atol=1e-13)
        th, m = nesterov_step(th, m, sum(gs) / N, 0.7, 0.9)
        np.testing.assert_allclose(dn.theta, th, atol=1e-12)
        np.testing.assert_allclose(dn.m, m, atol=1e-12)
        assert not dn.delta.any()


def test_dn_rejects_c_outside_range():
    with pytest.raises(ValueError):
        DelayedNesterov(np.zeros(2), 0.7, 0.9, 4, 0.5)
    with pytest.raises(ValueError):
        DelayedNesterov(np.zeros(2), 0.7, 0.9, 4, -0.1)


def test_pseudo_gradient_sign():
    a, b = np.array([1.0, 2.0]), np.array([0.5, 2.5])
    np.testing.assert_array_equal(pseudo_gradient(a, b), np.array([0.5, -0.5]))


# ----------------------------------------------------------------------------------- AdamW
def test_adamw_linear_loss_closed_form():
    # gradient g constant: bias-corrected m_hat = g and v_hat = g^2 at every step, so
    # theta <- (1 - lr wd) theta - lr g / (|g| + eps)
    g = np.array([0.3, -2.0, 1e-3])
    th = np.array([1.0, -1.0, 0.5])
    opt = AdamW(3, np.float64, wd=0.1)
    ref = th.copy()
    for _ in range(7):
        opt.step(th, g, 1e-2)
        ref = (1 - 1e-2 * 0.1) * ref - 1e-2 * g / (np.abs(g) + 1e-8)
        np.testing.assert_allclose(th, ref, rtol=1e-12)


def test_adamw_first_step_is_sign_of_gradient():
    g = np.array([5.0, -1e-3, 2.0])
    th = np.zeros(3)
    AdamW(3, np.float64, wd=0.0).step(th, g, 1e-3)
    np.testing.assert_allclose(th, -1e-3 * np.sign(g), rtol=1e-4)


def test_adamw_matches_library_on_quadratic_and_decay_mask():
    rng = np.random.default_rng(5)
    th0 = rng.standard_normal(6)
    A = rng.standard_normal((6, 6))
    A = A @ A.T + np.eye(6)
    # elements 0..3 decayed, 4..5 not: two library parameter groups
    p1 = torch.nn.Parameter(torch.tensor(th0[:4].copy()))
    p2 = torch.nn.Parameter(torch.tensor(th0[4:].copy()))
    lib = torch.optim.AdamW([dict(params=[p1], weight_decay=0.1), dict(params=[p2], weight_decay=0.0)],
                            lr=3e-3, betas=(0.9, 0.999), eps=1e-8)
    th = th0.copy()
    opt = AdamW(6, np.float64, wd=0.1, n_decayed=4)
    for _ in range(25):
        g = A @ th
        full = torch.cat([p1.detach(), p2.detach()]).numpy()
        gl = A @ full
        p1.grad, p2.grad = torch.tensor(gl[:4].copy()), torch.tensor(gl[4:].copy())
        lib.step()
        opt.step(th, g, 3e-3)
    np.testing.assert_allclose(th, torch.cat([p1.detach(), p2.detach()]).numpy(), rtol=1e-10, atol=1e-12)
    assert opt.n == 25


def test_adamw_scalar_quadratic_independent_loop():
    th, m, v = 2.0, 0.0, 0.0
    x = np.array([2.0])
    opt = AdamW(1, np.float64, wd=0.1)
    for n in range(1, 40):
        g = 3.0 * th
        m = 0.9 * m + 0.1 * g
        v = 0.999 * v + 0.001 * g * g
        th = th - 1e-2 * ((m / (1 - 0.9**n)) / (math.sqrt(v / (1 - 0.999**n)) + 1e-8) + 0.1 * th)
        opt.step(x, 3.0 * x, 1e-2)
        assert x[0] == pytest.approx(th, rel=1e-12)


# ------------------------------------------------------------------------------------ DyLU
def test_dylu_exact_counts(golden):
    G = golden("schedule_traces.txt")
    assert dylu_steps([1, 1.5, 2, 3], 5).tolist() == [int(x) for x in G["tiny_steps"]]
    assert dylu_steps([1, 1.2, 1.6, 2.4], 50).tolist() == [int(x) for x in G["lm20m_steps"]]
    assert dylu_steps([2.0, 2.0, 2.0], 7).tolist() == [7, 7, 7]


def test_dylu_proportional_to_speed_and_clamped():
    rng = np.random.default_rng(0)
    v = rng.uniform(1, 4, 16)
    H = 50
    s = dylu_steps(v, H)
    exact = v / v.max() * H
    assert np.all(s <= exact + 1e-9) and np.all(s > exact - 1)
    # completion times are within one step-time of the fastest worker's
    assert np.all(H / v.max() - s / v < 1.0 / v + 1e-12)
    assert dylu_steps([0.01, 10.0], 5).tolist() == [1, 5]
    with pytest.raises(ValueError):
        dylu_steps([1.0, -1.0], 5)
    with pytest.raises(ValueError):
        dylu_steps([1.0, float("nan")], 5)
    with pytest.raises(ValueError):
        dylu_steps([1.0], 0)


# ------------------------------------------------------------------------------- scheduler
def test_event_trace_tiny_hand_traced(golden):
    G = golden("schedule_traces.txt")
    steps = dylu_steps([1, 1.5, 2, 3], 5)
    ev = flat_events(event_trace([1, 1.5, 2, 3], steps, 0.0, 12))
    assert [e[0] for e in ev] == [int(x) for x in G["tiny_workers"]]
    assert [e[1] for e in ev] == G["tiny_times"]          # bit-exact fp64
    assert [e[2] for e in ev] == [int(x) for x in G["tiny_group_end"]]


def test_event_trace_lm20m_tie_group(golden):
    G = golden("schedule_traces.txt")
    v = [1, 1.2, 1.6, 2.4]
    ev = flat_events(event_trace(v, dylu_steps(v, 50), 0.0, 4))
    assert [e[0] for e in ev] == [int(x) for x in G["lm20m_workers"]]
    assert [e[2] for e in ev] == [int(x) for x in G["lm20m_group_end"]]
    assert ev[2][1] == ev[3][1] == 25 / 1.2 == 50 / 2.4


def test_event_trace_equal_speeds_groups_of_k():
    groups = event_trace([2.0] * 3, [4] * 3, 0.0, 9)
    assert [[w for w, _ in g["events"]] for g in groups] == [[0, 1, 2]] * 3
    assert [g["events"][0][1] for g in groups] == [2.0, 4.0, 6.0]


def test_event_trace_grace_window_groups_and_delays_restart():
    # B finishes 0.3 after A (inside a 0.5 window): same group, both restart at A + 0.5;
    # C finishes 1.0 after A: starts its own window.  (Grace-period figure caption.)
    v = [1.0, 1.0, 1.0]
    groups = event_trace(v, [10, 10, 10], 0.5, 3)        # identical: one group at t=10
    assert [w for w, _ in groups[0]["events"]] == [0, 1, 2]
    groups = event_trace([10 / 10.0, 10 / 10.3, 10 / 11.0], [10, 10, 10], 0.5, 5)
    assert [[w for w, _ in g["events"]] for g in groups[:2]] == [[0, 1], [2]]
    assert groups[0]["restart_time"] == pytest.approx(10.5)
    assert groups[1]["restart_time"] == pytest.approx(11.5)
    # after the restart A and B finish together at 20.5 and 20.8 -> grouped again
    assert [w for w, _ in groups[2]["events"]] == [0, 1]
    assert groups[2]["events"][0][1] == pytest.approx(20.5)


def test_event_trace_cut_mid_group_is_flagged():
    groups = event_trace([1.0, 1.0], [2, 2], 0.0, 3)
    assert groups[-1]["complete"] is False and len(groups[-1]["events"]) == 1
    groups = event_trace([1.0, 1.0], [2, 2], 0.0, 4)
    assert groups[-1]["complete"] is True and len(groups) == 2


# ------------------------------------------------- comparison rules ("Existing Fixes")
def test_poly_weight_values():
    from oracle.optim import poly_weight
    assert poly_weight(0) == 1.0
    assert poly_weight(3) == pytest.approx(0.5)
    assert poly_weight(8) == pytest.approx(1.0 / 3.0)
    assert poly_weight(3, 1.0) == pytest.approx(0.25)


def test_delay_compensation_formula_and_identity():
    from oracle.optim import delay_compensated
    g = np.array([2.0, -1.0, 0.0])
    now, then = np.array([1.0, 1.0, 5.0]), np.array([0.5, 2.0, 0.0])
    np.testing.assert_array_equal(delay_compensated(g, now, then, 0.0), g)
    # g + lam g^2 (now - then): 2 + .1*4*.5 = 2.2 ; -1 + .1*1*(-1) = -1.1 ; 0
    np.testing.assert_allclose(delay_compensated(g, now, then, 0.1), [2.2, -1.1, 0.0], atol=1e-15)
    np.testing.assert_array_equal(delay_compensated(g, then, then, 7.0), g)       # no drift, no correction


def test_async_buffer_is_nesterov_on_the_mean_and_matches_dn_at_period_ends():
    from oracle.optim import AsyncBuffer
    rng = np.random.default_rng(4)
    N = 4
    th0 = rng.standard_normal(6)
    buf = AsyncBuffer(th0, 0.7, 0.9, N)
    dn = DelayedNesterov(th0, 0.7, 0.9, N, 0.0)
    th, m = th0.copy(), np.zeros(6)
    for _ in range(3):
        gs = [rng.standard_normal(6) for _ in range(N)]
        before = buf.theta.copy()
        for j, g in enumerate(gs):
            buf.event(g)
            dn.event(g)
            if j < N - 1:
                np.testing.assert_array_equal(buf.theta, before)       # parameters wait for the buffer
        th, m = nesterov_step(th, m, sum(gs) / N, 0.7, 0.9)
        np.testing.assert_allclose(buf.theta, th, atol=1e-12)
        np.testing.assert_allclose(buf.m, m, atol=1e-12)
        # with the same pseudo-gradients Delayed Nesterov (c = 0) lands on the same point every N events
        np.testing.assert_allclose(dn.theta, buf.theta, atol=1e-12)
    b1 = AsyncBuffer(th0, 0.7, 0.9, 1)                                   # N = 1 is plain Nesterov
    th, m = th0.copy(), np.zeros(6)
    for _ in range(4):
        g = rng.standard_normal(6)
        b1.event(g)
        th, m = nesterov_step(th, m, g, 0.7, 0.9)
        np.testing.assert_allclose(b1.theta, th, atol=1e-13)
