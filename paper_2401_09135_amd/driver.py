"""Driver for a whole asynchronous run: asks the library for DyLU step counts and the event
order (als_dylu_schedule), then issues als_worker_local_steps / als_outer_apply_dn calls in
that order.  It holds no arithmetic of the method: every update runs in the library."""
from __future__ import annotations

import numpy as np

from .binding import Config, Context, dylu_schedule


def run_async(w: dict, theta0: np.ndarray, make_stream, n_events: int | None = None, flags: int = 0,
              ctx: Context | None = None, collect_losses: bool = True, lr=None, rule: dict | None = None,
              on_group=None):
    """w: workload dict (als_inputs.workload); make_stream(i) -> object with take(n) giving
    int32 [n,B,S+1] token batches for worker i.  Returns dict like the oracle's run.
    on_group(ctx, index of the group's last event): optional observer called after every applied
    group of sync events (before its workers are given new rounds)."""
    import torch
    n_events = w["n_events"] if n_events is None else n_events
    steps, ev_w, ev_t, ev_g = dylu_schedule(w["speeds"], w["H"], w["tau_grace"], n_events)
    own = ctx is None
    if own:
        cfg = Config.from_workload(w, flags=flags, max_local_steps=int(steps.max()))
        ctx = Context(cfg, theta0)
    k = w["k"]
    streams = [make_stream(i) for i in range(k)]
    losses = [[] for _ in range(k)]
    pending = [0] * k
    lr = w["lr"] if lr is None else lr

    def train(i):
        tok = torch.from_numpy(streams[i].take(int(steps[i]))).to(ctx.device)
        ctx.worker_local_steps(i, tok, lr)
        pending[i] = int(steps[i])

    def harvest(i):
        if collect_losses and pending[i]:
            losses[i].extend(ctx.get_losses(i, pending[i]).tolist())
        pending[i] = 0

    for i in range(k):
        train(i)
    e = 0
    while e < n_events:
        j = e
        while j < n_events - 1 and not ev_g[j]:
            j += 1
        group = [int(x) for x in ev_w[e:j + 1]]
        complete = bool(ev_g[j])
        for i in group:
            harvest(i)
        if rule:
            ctx.outer_apply_rule(group, restart=complete, **rule)
        else:
            ctx.outer_apply_dn(group, restart=complete)
        if on_group is not None:
            on_group(ctx, j)
        if complete and j + 1 < n_events:
            for i in group:
                train(i)
        e = j + 1
    ctx.sync()
    for i in range(k):
        harvest(i)
    out = dict(theta=ctx.get_vector("theta"), m=ctx.get_vector("momentum"), delta=ctx.get_vector("delta"),
               t=ctx.server_t, losses=losses, steps=steps, ev_worker=ev_w, ev_time=ev_t, ev_group_end=ev_g, ctx=ctx)
    return out
