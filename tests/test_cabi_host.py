"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host
logic (DyLU, event order, layout, argument validation) agrees bit for bit with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

import als_inputs as I
import paper_2401_09135_amd as A
from oracle import lm
from oracle.optim import dylu_steps
from oracle.scheduler import event_trace, flat_events

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "als.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(als_[a-z0-9_]+)\s*\(", hdr)))
    assert {"als_init", "als_worker_local_steps", "als_outer_apply_dn", "als_dylu_schedule"} <= set(names)
    lib = ctypes.CDLL(A.lib_path)
    for n in names:
        assert hasattr(lib, n), n


@pytest.mark.parametrize("name", list(I.WORKLOADS))
def test_layout_agrees_with_oracle(name):
    w = I.workload(name)
    cfg = A.Config.from_workload(w)
    lay = lm.param_layout(w)
    assert A.param_count(cfg) == lm.n_params(w)
    assert A.param_count_decayed(cfg) == lm.n_decayed(w)
    offs, off = [], 0
    for _n, shape, _k in lay:
        offs.append(off)
        off += int(np.prod(shape))
    assert A.param_offsets(cfg).tolist() == offs


def _trace_from_lib(v, H, grace, n):
    steps, ew, et, eg = A.dylu_schedule(v, H, grace, n)
    return steps.tolist(), list(zip(ew.tolist(), et.tolist(), eg.tolist()))


@pytest.mark.parametrize("name", list(I.WORKLOADS))
def test_schedule_bit_exact_on_workloads(name):
    w = I.workload(name)
    n = 5 * w["k"]
    steps, ev = _trace_from_lib(w["speeds"], w["H"], w["tau_grace"], n)
    osteps = dylu_steps(w["speeds"], w["H"])
    assert steps == osteps.tolist()
    assert ev == flat_events(event_trace(w["speeds"], osteps, w["tau_grace"], n))


def test_schedule_bit_exact_random_speeds_ties_and_grace():
    rng = np.random.default_rng(0)
    for trial in range(200):
        k = int(rng.integers(1, 17))
        if trial % 3 == 0:      # many exact ties
            v = rng.choice([1.0, 1.5, 2.0, 3.0, 4.0], size=k)
        else:
            v = rng.uniform(0.2, 4.0, size=k)
        H = int(rng.integers(1, 60))
        grace = float(rng.choice([0.0, 0.0, 0.25, 1.0, 3.0]))
        n = int(rng.integers(1, 80))
        steps, ev = _trace_from_lib(v, H, grace, n)
        osteps = dylu_steps(v, H)
        assert steps == osteps.tolist(), (trial, v, H)
        assert ev == flat_events(event_trace(v, osteps, grace, n)), (trial, v, H, grace, n)


def test_schedule_without_trace_and_errors():
    steps, ew, _, _ = A.dylu_schedule([1, 1.5, 2, 3], 5)
    assert steps.tolist() == [1, 2, 3, 5] and ew.size == 0
    assert A.dylu_schedule([0.001, 5.0], 10)[0].tolist() == [1, 10]      # clamped to one step
    for bad in ([], [1.0, 0.0], [1.0, -2.0], [float("nan")], [float("inf")]):
        with pytest.raises(A.AlsError):
            A.dylu_schedule(bad, 5)
    with pytest.raises(A.AlsError):
        A.dylu_schedule([1.0], 0)
    with pytest.raises(A.AlsError):
        A.dylu_schedule([1.0], 5, -1.0, 3)
    with pytest.raises(A.AlsError):
        A.dylu_schedule(np.ones(65), 5)


def test_config_validation():
    good = I.workload("tiny")
    assert A.param_count(A.Config.from_workload(good)) > 0
    for key, val in [("d", 96), ("h", 3), ("ff", 100), ("S", 2000), ("k", 0), ("N", 0), ("V", 1),
                     ("dn_c", 0.5), ("beta1", 1.0), ("norm_eps", 0.0), ("B", 0)]:
        bad = dict(good)
        bad[key] = val
        cfg = A.Config.from_workload(bad)
        assert A.param_count(cfg) == 0, key
        assert A.lib.als_arena_bytes(ctypes.byref(cfg)) == 0, key
        assert A.lib.als_last_error()      # a message was left
