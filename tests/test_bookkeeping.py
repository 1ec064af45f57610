"""train() bookkeeping (Eq. lr, Eq. data_sample): oracle pins and library agreement (CPU only)."""
import math

import numpy as np
import pytest

import paper_2401_09135_amd as A
from oracle.bookkeeping import lr_schedule, shard_probabilities, shard_sample


# ------------------------------------------------------------------------------ oracle pins
def test_lr_schedule_closed_forms():
    W, T, hi, lo = 1000, 64000, 1e-3, 1e-6        # the paper's warm-up and final inner lr
    assert lr_schedule(0, W, T, hi, lo) == 0.0
    assert lr_schedule(500, W, T, hi, lo) == pytest.approx(0.5e-3, rel=1e-15)      # linear warm-up
    assert lr_schedule(W, W, T, hi, lo) == pytest.approx(hi, rel=1e-15)            # continuous at t_warmup
    assert lr_schedule((W + T) // 2, W, T, hi, lo) == pytest.approx((hi + lo) / 2, rel=1e-12)   # cos(pi/2) = 0
    assert lr_schedule(T, W, T, hi, lo) == pytest.approx(lo, rel=1e-12)
    assert lr_schedule(10 * T, W, T, hi, lo) == pytest.approx(lo, rel=1e-12)       # ratio clamped: eta_min beyond T
    # quarter point: cos(pi/4) = sqrt(2)/2
    q = W + (T - W) // 4
    assert lr_schedule(q, W, T, hi, lo) == pytest.approx(lo + 0.5 * (hi - lo) * (1 + math.sqrt(0.5)), rel=1e-12)
    # degenerate horizons: T <= t_warmup gives eta_min right after the warm-up
    assert lr_schedule(5, 5, 5, hi, lo) == pytest.approx(lo)
    assert lr_schedule(7, 5, 3, hi, lo) == pytest.approx(lo)
    # no warm-up
    assert lr_schedule(0, 0, 100, hi, lo) == pytest.approx(hi)
    vals = [lr_schedule(t, W, T, hi, lo) for t in range(W, T + 1, 777)]
    assert all(a >= b for a, b in zip(vals, vals[1:]))                              # monotone decay


def test_lr_schedule_matches_library_cosine_annealing():
    torch = pytest.importorskip("torch")
    W, T, hi, lo = 0, 50, 1e-2, 1e-4
    p = torch.nn.Parameter(torch.zeros(1))
    opt = torch.optim.SGD([p], lr=hi)
    sch = torch.optim.lr_scheduler.CosineAnnealingLR(opt, T_max=T, eta_min=lo)
    for t in range(T + 1):
        assert opt.param_groups[0]["lr"] == pytest.approx(lr_schedule(t, W, T, hi, lo), rel=1e-9)
        opt.step()
        sch.step()


def test_shard_probabilities_hand_worked():
    # size shares (.25, .25, .5); progress shares (.5, 0, .5): only the middle shard is behind
    np.testing.assert_allclose(shard_probabilities([1, 1, 2], [10, 0, 10]), [0, 1, 0])
    # nothing learned yet: the size shares
    np.testing.assert_allclose(shard_probabilities([1, 1, 2], [0, 0, 0]), [0.25, 0.25, 0.5])
    # exactly on target everywhere: falls back to the size shares
    np.testing.assert_allclose(shard_probabilities([1, 3], [5, 15]), [0.25, 0.75])
    # shares (.5,.3,.2), progress (.2,.3,.5): differences (.3, 0, -.3) -> (1, 0, 0)
    np.testing.assert_allclose(shard_probabilities([5, 3, 2], [2, 3, 5]), [1, 0, 0], atol=1e-15)
    # shares (.4,.4,.2), progress (.1,.3,.6): (.3,.1,0) -> (.75,.25,0)
    np.testing.assert_allclose(shard_probabilities([2, 2, 1], [1, 3, 6]), [0.75, 0.25, 0], atol=1e-15)
    with pytest.raises(ValueError):
        shard_probabilities([1, 0], [0, 0])
    with pytest.raises(ValueError):
        shard_probabilities([1, 1], [0, -1])


def test_shard_sampling_balances_progress():
    # sampling by Eq. (data_sample) and crediting one unit per draw drives progress to the size shares
    rng = np.random.default_rng(0)
    sizes = np.array([1.0, 2.0, 5.0])
    learned = np.array([30.0, 0.0, 0.0])
    for _ in range(4000):
        learned[shard_sample(sizes, learned, rng.random())] += 1
    np.testing.assert_allclose(learned / learned.sum(), sizes / sizes.sum(), atol=0.01)
    # inverse CDF: u just below / above a boundary
    assert shard_sample([2, 2, 1], [1, 3, 6], 0.7499) == 0 and shard_sample([2, 2, 1], [1, 3, 6], 0.7501) == 1


# ------------------------------------------------------------------ library agrees with oracle
def test_library_lr_schedule_matches_oracle():
    for (W, T, hi, lo) in [(1000, 64000, 1e-3, 1e-6), (0, 100, 0.1, 0.0), (10, 10, 1e-3, 1e-6), (50, 20, 1e-3, 2e-4)]:
        got = A.lr_schedule(0, 300, W, T, hi, lo)
        ref = np.array([lr_schedule(t, W, T, hi, lo) for t in range(300)], dtype=np.float64)
        np.testing.assert_allclose(got, ref.astype(np.float32), rtol=2e-7, atol=1e-12)
    got = A.lr_schedule(63990, 20, 1000, 64000, 1e-3, 1e-6)
    ref = np.array([lr_schedule(t, 1000, 64000, 1e-3, 1e-6) for t in range(63990, 64010)])
    np.testing.assert_allclose(got, ref.astype(np.float32), rtol=2e-7)
    assert A.lr_schedule(5, 0, 1, 2, 1.0, 0.0).size == 0
    for bad in [(-1, 1, 0, 10, 1.0, 0.0), (0, 1, 0, 10, 1.0, 2.0), (0, 1, 0, 10, float("nan"), 0.0)]:
        with pytest.raises(A.AlsError):
            A.lr_schedule(*bad)


def test_library_shard_sample_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(300):
        k = int(rng.integers(1, 9))
        sizes = rng.uniform(0.5, 5.0, k)
        learned = rng.integers(0, 50, k).astype(np.float64) * (rng.random() > 0.2)
        u = float(rng.random())
        p, pick = A.shard_sample(sizes, learned, u)
        np.testing.assert_allclose(p, shard_probabilities(sizes, learned), rtol=1e-14, atol=1e-16)
        assert pick == shard_sample(sizes, learned, u)
    with pytest.raises(A.AlsError):
        A.shard_sample([1.0, -1.0], [0.0, 0.0], 0.5)
    with pytest.raises(A.AlsError):
        A.shard_sample([1.0], [0.0], 1.0)
