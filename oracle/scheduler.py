"""Asynchronous task scheduling on a simulated clock -- Alg. 2 with get_worker() from the
appendix pseudocode, made deterministic the way the Async. Local-SGD Framework section
describes (faked training time from device speed).

Readings where the paper is silent: a job of H_i steps on a worker of speed v_i (steps per
second) lasts H_i / v_i; the outer step and the model copies take no simulated time; the
"earliest completed worker" under exact ties is the one with the smaller index; workers
released together restart at tau_sync + tau_grace, the moment the server knows nobody else
arrives inside the window; the loop stops after a fixed number of sync events.
"""
from __future__ import annotations

import math
import numpy as np


def event_trace(speeds, steps, tau_grace, n_events):
    """Returns a list of groups; each group is a dict
         {"events": [(worker, completed_time), ...], "restart_time": float}
    in the order the server processes them.  After the last requested event the loop looks
    one decision ahead: if the next worker would still join the open group, the group is
    cut short and its "complete" flag is False (no restart follows)."""
    v = np.asarray(speeds, dtype=np.float64)
    H = np.asarray(steps, dtype=np.int64)
    k = v.size
    start = np.zeros(k, dtype=np.float64)
    done = np.array([start[i] + float(H[i]) / v[i] for i in range(k)], dtype=np.float64)
    running = [True] * k            # has an unprocessed result pending
    completed = []                  # W_completed
    tau_sync = math.inf
    groups, cur, emitted = [], [], 0
    while True:
        cand = [i for i in range(k) if running[i]]
        w = None
        if cand:
            e = min(cand, key=lambda i: (done[i], i))
            if math.isinf(tau_sync) or done[e] - tau_sync <= tau_grace:
                w = e
        if w is not None:
            if emitted == n_events:         # the event budget cuts this group short
                groups.append(dict(events=cur, restart_time=float(tau_sync + tau_grace),
                                   complete=False))
                break
            tau_sync = min(tau_sync, done[w])
            cur.append((int(w), float(done[w])))
            running[w] = False
            completed.append(w)
            emitted += 1
        else:
            restart = tau_sync + tau_grace
            groups.append(dict(events=cur, restart_time=float(restart), complete=True))
            for i in completed:
                start[i] = restart
                done[i] = start[i] + float(H[i]) / v[i]
                running[i] = True
            completed, cur, tau_sync = [], [], math.inf
            if emitted == n_events:
                break
    return groups


def flat_events(groups):
    """[(worker, time, group_end_flag)] in processing order."""
    out = []
    for g in groups:
        n = len(g["events"])
        for j, (w, t) in enumerate(g["events"]):
            out.append((w, t, 1 if (j == n - 1 and g["complete"]) else 0))
    return out
