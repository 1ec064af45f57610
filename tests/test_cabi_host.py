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
    # the internal measurement / tuning hooks (not part of the ABI) are exported as declared too
    hooks = open(os.path.join(ROOT, "paper_2401_09135_amd", "csrc", "als_bench.h")).read()
    hooks = re.sub(r"/\*.*?\*/", "", hooks, flags=re.S)
    hook_names = sorted(set(re.findall(r"\b(als_[a-z0-9_]+)\s*\(", hooks)))
    assert "als_k_gemm_dw_grouped_plan" in hook_names
    for n in hook_names:
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


def _dw_plan(Ms, Ns, K):
    n = len(Ms)
    fn = A.lib.als_k_gemm_dw_grouped_plan
    fn.restype = ctypes.c_int
    I32 = ctypes.POINTER(ctypes.c_int32)
    fn.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int), ctypes.c_int,
                   ctypes.c_int, I32, ctypes.c_int, I32, I32]
    counts = np.zeros(6, np.int32)
    Mc, Nc = (ctypes.c_int * n)(*Ms), (ctypes.c_int * n)(*Ns)
    rc = fn(n, Mc, Nc, K, 0, None, 0, None, counts.ctypes.data_as(I32))
    if rc:
        return rc, None, None, None
    items = np.zeros((max(int(counts[0]), 1), 6), np.int32)
    split = np.zeros((max(int(counts[1]), 1), 5), np.int32)
    rc = fn(n, Mc, Nc, K, len(items), items.ctypes.data_as(I32), len(split), split.ctypes.data_as(I32),
            counts.ctypes.data_as(I32))
    assert rc == 0
    return 0, items[: counts[0]], split[: counts[1]], counts


def _lm_dw_shapes(name):
    w = I.workload(name)
    d, ff, a = w["d"], w["ff"], w["h"] * (w.get("dh") or w["d"] // w["h"])
    per_layer = [(ff, d), (d, ff), (a, d), (d, 3 * a)]
    return per_layer * w["L"], w["B"] * w["S"]


_DW_CASES = [([128], [128], 64), ([256], [256], 256), ([896, 3584, 896, 896], [3584, 896, 896, 2688], 16384),
             ([128] * 7, [384] * 7, 1024), ([256] * 300, [256] * 300, 512), ([1152], [640], 192),
             ([2048] * 16, [2048] * 16, 128), ([768] * 50, [768] * 50, 128), ([896, 3584] * 6, [3584, 896] * 6, 256), ([512, 2048, 512, 512] * 6, [2048, 512, 512, 1536] * 6, 16384)]


@pytest.mark.parametrize("Ms,Ns,K", _DW_CASES + [(*map(list, zip(*_lm_dw_shapes(n)[0])), _lm_dw_shapes(n)[1])
                                                 for n in ("lm150m", "lm20m", "paper60m")])
def test_grouped_weight_gradient_plan_covers_every_tile_and_slice_once(Ms, Ns, K):
    """The work-item list of the grouped weight-gradient launch, rebuilt by brute force: every
    256 x 256 tile of every product has every 64-wide K slice exactly once; a tile is either one
    whole item that writes the gradient (slot -1) or a set of K-split items with distinct slots that
    the split-tile table lists in full; everything stays inside the tables and the partial-tile
    buffer the workspace provides."""
    rc, items, split, counts = _dw_plan(Ms, Ns, K)
    assert rc == 0
    n_items, n_split, n_partial, cap_items, cap_split, cap_slots = (int(c) for c in counts)
    nk = K // 64
    tiles = {(p, tm, tn) for p, (m, n) in enumerate(zip(Ms, Ns)) for tm in range(-(-m // 256)) for tn in range(-(-n // 256))}
    assert n_items <= cap_items and n_split <= cap_split and n_partial <= cap_slots
    cover = {t: np.zeros(nk, np.int32) for t in tiles}
    whole, parts, slots = set(), {}, []
    for p, tm, tn, slot, s0, cnt in items.tolist():
        assert (p, tm, tn) in tiles and cnt >= 1 and 0 <= s0 and s0 + cnt <= nk
        cover[(p, tm, tn)][s0:s0 + cnt] += 1
        if slot < 0:
            assert s0 == 0 and cnt == nk
            whole.add((p, tm, tn))
        else:
            assert 0 <= slot < n_partial
            slots.append(slot)
            parts.setdefault((p, tm, tn), []).append(slot)
    for t, c in cover.items():
        assert (c == 1).all(), t
    assert not (whole & set(parts)) and len(whole) + len(parts) == len(tiles)
    assert sorted(slots) == list(range(n_partial))
    assert len(parts) == n_split
    listed = {}
    for p, tm, tn, slot0, nslots in split.tolist():
        assert (p, tm, tn) not in listed
        listed[(p, tm, tn)] = list(range(slot0, slot0 + nslots))
    assert {t: sorted(s) for t, s in parts.items()} == listed
    # the chip is filled: whole tiles come in full rounds of the CU count unless nothing is split
    if n_split:
        assert len(whole) % cap_slots == 0 and n_items - len(whole) <= cap_slots


def test_grouped_weight_gradient_plan_rejects_unsupported_shapes():
    for Ms, Ns, K in [([100], [128], 64), ([128], [192], 64), ([128], [128], 96), ([128], [128], 0), ([0], [128], 64)]:
        rc, *_ = _dw_plan(Ms, Ns, K)
        assert rc == -1   # ALS_ERR_INVALID
