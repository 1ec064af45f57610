"""Writes the full-size one-outer-round fixtures tests/golden/round_<workload>.npz.

Calls only the CPU oracle (oracle/) and the seeded input recipes (als_inputs): nothing here
touches the HIP library, so every stored value is the oracle's.

One outer round = N consecutive sync events of Alg. 2 (one Delayed-Nesterov period, Alg. 3),
at the workload's full model shapes and batch.  The fastest worker's step count H (Eq. DyLU) can
be lowered with --H so that the fp32 numpy oracle finishes in an hour on a handful of cores; the
value used is stored in the fixture and the GPU test reads it from there.

Stored per workload:
  H, n_events, steps [k], ev_worker / ev_time [n_events]      the schedule (bit-exact quantities)
  loss_<i> [steps run by worker i]                             every per-step loss
  idx [n]                                                      sampled flat indices (per tensor, strided)
  theta [n], m [n], delta [n]                                  server vectors on the sample, after the round
  theta_ev [n_events, n_ev] on idx[::ev_stride]                server parameters after each event
  tnorm_theta / tnorm_m / tnorm_upd [n_tensors]                per-tensor L2 norms of theta, m, theta - theta0
                                                               over the WHOLE tensor (float64 accumulation)

usage: python tests/golden/make_full_size_round.py lm20m [--H 50] [--per-tensor 4096]
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import als_inputs as I          # noqa: E402
from oracle import lm, run      # noqa: E402


def sample_indices(w, per_tensor):
    """Strided sample of every tensor of the flat layout: at most per_tensor elements each, the
    stride odd so that it walks across rows and columns."""
    idx, off = [], 0
    for _name, shape, _kind in lm.param_layout(w):
        n = int(np.prod(shape))
        stride = max(1, n // per_tensor) | 1
        idx.append(off + np.arange(0, n, stride, dtype=np.int64)[:per_tensor])
        off += n
    return np.concatenate(idx)


def tensor_norms(v, w):
    out, off = [], 0
    for _name, shape, _kind in lm.param_layout(w):
        n = int(np.prod(shape))
        out.append(float(np.sqrt(np.sum(np.square(v[off:off + n], dtype=np.float64)))))
        off += n
    return np.asarray(out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("workload")
    ap.add_argument("--H", type=int, default=None)
    ap.add_argument("--per-tensor", type=int, default=4096)
    ap.add_argument("--ev-stride", type=int, default=4)
    ap.add_argument("--out", default=None)
    ap.add_argument("--progress-every", type=int, default=4)
    a = ap.parse_args()
    w = I.workload(a.workload)
    if a.H is not None:
        w["H"] = a.H
    n_events = w["N"]                      # one outer round
    theta0 = I.theta0(lm.param_layout(w), w["seed"])
    idx = sample_indices(w, a.per_tensor)
    ev_idx = idx[::a.ev_stride]
    theta_ev = []
    t0 = time.time()

    def log(server, wi):
        theta_ev.append(server.theta[ev_idx].copy())
        print(f"[{time.time() - t0:8.0f} s] event {server.t} (worker {wi}) applied", flush=True)

    class Stream(I.TokenStream):           # progress line per batch request (a worker's local round)
        def take(self, n):
            print(f"[{time.time() - t0:8.0f} s] worker round of {n} steps starts", flush=True)
            return super().take(n)

    # a progress line every few local steps (the oracle's own loss-and-gradient routine, counted)
    inner, count = lm.loss_and_grad, [0]

    def counted(theta, tokens, cfg):
        out = inner(theta, tokens, cfg)
        count[0] += 1
        if count[0] % a.progress_every == 0:
            print(f"[{time.time() - t0:8.0f} s] {count[0]} local steps done, last loss {float(out[0]):.4f}", flush=True)
        return out
    lm.loss_and_grad = counted

    ref = run.run_async(w, theta0, lambda i: Stream(w["seed"], i, w["B"], w["S"], w["V"]),
                        n_events=n_events, log=log)
    lm.loss_and_grad = inner
    ev = [(wk, t) for g in ref["groups"] for (wk, t) in g["events"]]
    out = dict(H=np.int64(w["H"]), n_events=np.int64(n_events), steps=np.asarray(ref["steps"], np.int64),
               ev_worker=np.asarray([e[0] for e in ev], np.int64), ev_time=np.asarray([e[1] for e in ev], np.float64),
               idx=idx, ev_stride=np.int64(a.ev_stride),
               theta=ref["theta"][idx], m=ref["m"][idx], delta=ref["delta"][idx],
               theta_ev=np.stack(theta_ev),
               tnorm_theta=tensor_norms(ref["theta"], w), tnorm_m=tensor_norms(ref["m"], w),
               tnorm_upd=tensor_norms(ref["theta"] - theta0, w))
    for i, l in enumerate(ref["losses"]):
        out[f"loss_{i}"] = np.asarray(l, np.float64)
    path = a.out or os.path.join(ROOT, "tests", "golden", f"round_{a.workload}.npz")
    np.savez_compressed(path, **out)
    print(f"wrote {path}: {os.path.getsize(path) / 1e6:.2f} MB, {time.time() - t0:.0f} s", flush=True)


if __name__ == "__main__":
    main()
