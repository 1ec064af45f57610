"""Benchmark of the asynchronous Local-SGD hot path on one MI355X.

A "step" is one outer round of the paper's asynchronous schedule on the 20M-class workload:
N = 4 sync events (pseudo-gradient + Delayed Nesterov + restart) together with the local rounds
(DyLU step counts 20/25/33/50, each step = forward + backward + AdamW on 32 x 512 tokens) of the
four simulated workers, which run on their own HIP streams.  Tokens are synthetic Zipf(1.1)
draws, resident in HBM before the clock starts.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E
# HBM bytes per launch of the step's GEMM kernels, measured with rocprofv3 --pmc FETCH_SIZE (x 2.0)
# and WRITE_SIZE (x 1.0) on the same shapes (profiles/gemm_mfma_microbench.md gives the commands,
# the calibration of the two factors and the comparison with the algorithmic bytes).  Counters
# cannot be collected from inside this process, so the figure is carried here.
MEASURED_TRAFFIC_BYTES = {"lm20m": {"gemm_mfma_kernel<128, 128, 1, 0, STORE, float, true, 2, 2>": 99.0e6}}


def flops_per_token(w):
    """Algorithmic training FLOPs per token: 3 x [L (8 d a + 4 d ff + 2 S a) + 2 d V], a = attention
    width (= d unless the workload sets a head width); causal attention counted at half, backward
    = 2 x forward, no recompute credit.  With a = d and ff = 4 d this is 3 [L (24 d^2 + 2 S d) + 2 d V]."""
    L, d, S, V, ff = w["L"], w["d"], w["S"], w["V"], w["ff"]
    a = w["h"] * w["dh"] if w.get("dh") else d
    return 3.0 * (L * (8.0 * d * a + 4.0 * d * ff + 2.0 * S * a) + 2.0 * d * V)


def _host_threads():
    """(threads the BLAS behind numpy uses, its name)."""
    try:
        from threadpoolctl import threadpool_info
        info = [p for p in threadpool_info() if p.get("user_api") == "blas"] or threadpool_info()
        return max([p.get("num_threads", 1) for p in info] or [1]), "/".join(
            sorted({f"{p.get('internal_api', '?')} {p.get('version', '')}".strip() for p in info})) or "unknown"
    except Exception:
        return os.cpu_count() or 1, "unknown"


def cpu_baseline_outer(mb):
    """The oracle's Delayed Nesterov event (pseudo-gradient + Alg. 3, numpy fp32) on the same
    150M-element vectors: two non-boundary events timed, 24 algorithmic bytes per parameter."""
    import numpy as np
    import als_inputs as I
    from oracle.optim import DelayedNesterov, pseudo_gradient
    P = mb["P"]
    rng = np.random.default_rng(mb["seed"])
    theta = (rng.standard_normal(P, dtype=np.float32) * np.float32(mb["sigma"]))
    start = (rng.standard_normal(P, dtype=np.float32) * np.float32(mb["sigma"]))
    work = start + rng.standard_normal(P, dtype=np.float32) * np.float32(mb["drift_sigma"])
    server = DelayedNesterov(theta, mb["outer_lr"], mb["outer_beta"], 4, 0.0)
    t0 = time.perf_counter()
    n = 2
    for _ in range(n):
        server.event(pseudo_gradient(start, work))
    dt = (time.perf_counter() - t0) / n
    return dict(value=P * 24 / dt / 1e9, unit="GB/s", cores=1, kind="oracle",
                sample=f"{n} non-boundary Delayed-Nesterov events (N=4, c=0) on {P} fp32 parameters, numpy "
                       f"elementwise arithmetic (single-threaded), {dt:.2f} s per event on {os.cpu_count()} host cpus")


def cpu_baseline(w, seconds_hint=20.0):
    """The oracle as it stands, timed on the host: one local step (forward, backward, AdamW) of
    worker 0 on a slice of its batch, sized to take roughly 10-30 s."""
    import numpy as np
    import als_inputs as I
    from oracle import lm
    from oracle.optim import AdamW
    threads, blas = _host_threads()
    nb = max(1, w["B"] // 8)
    toks = I.TokenStream(w["seed"], 0, w["B"], w["S"], w["V"]).take(6)
    while True:
        theta = I.theta0(lm.param_layout(w), w["seed"])
        opt = AdamW(theta.size, np.float32, w["beta1"], w["beta2"], w["adam_eps"], w["wd"], lm.n_decayed(w))
        n, t0 = 0, time.perf_counter()
        while True:             # whole steps on the sample until about 10 s are spent (6 at most)
            _loss, grad = lm.loss_and_grad(theta, toks[n][:nb], w)
            opt.step(theta, grad, w["lr"])
            n += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or n == 6 or (n == 1 and dt < 2.5 and nb < w["B"]):
                break
        if dt >= 8.0 or nb >= w["B"]:
            break
        nb = min(w["B"], nb * 4)      # grow the sample until it is worth about 10-30 s
    return dict(value=n * nb * w["S"] / dt, unit="tokens/s", cores=int(threads), kind="oracle",
                sample=f"{n} local step(s) (forward+backward+AdamW, numpy fp32) of worker 0 on {nb} of its "
                       f"{w['B']} sequences of {w['S']} tokens; {dt:.1f} s on {os.cpu_count()} host cpus, "
                       f"BLAS {blas} with {threads} threads")


def outer_microbench(args):
    """Benchmark configs[2]: pseudo-gradient + Delayed Nesterov (single events, the grouped pass with
    fused restart) and fused AdamW on a 150M-element fp32 vector; achieved HBM GB/s from the
    algorithmic bytes per parameter (DN: 24 non-boundary, 32 boundary, grouped G events with
    restart 8G + 24 + 10G; AdamW: 30 with fp32 gradient and bf16 copy)."""
    import numpy as np
    import torch
    import als_inputs as I
    import paper_2401_09135_amd as A
    mb = I.OUTER_MICROBENCH
    P, dev = mb["P"], "cuda:0"
    G = 16
    gen = torch.Generator(device=dev).manual_seed(mb["seed"])
    rnd = lambda s: torch.randn(P, device=dev, generator=gen) * s
    theta, m, delta = rnd(mb["sigma"]), rnd(1e-3), torch.zeros(P, device=dev)
    starts = [rnd(mb["sigma"]) for _ in range(G)]
    works = [s + rnd(mb["drift_sigma"]) for s in starts]
    lps = [torch.empty(P, dtype=torch.bfloat16, device=dev) for _ in range(G)]

    def timed(fn, iters):
        for i in range(2):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    iters = max(args.steps, 20)
    res = {}
    # single events rotating over the 16 replicas so that nothing stays in the last-level cache
    for label, N, t0, bpp in (("dn_event_nonboundary_N4", 4, 0, 24), ("dn_event_boundary_N4", 4, 3, 32),
                              ("dn_event_N1_nesterov", 1, 0, 32), ("dn_event_nonboundary_N8", 8, 0, 24)):
        ms = timed(lambda i: A.k_dn_group(theta, m, delta, [starts[i % G]], [works[i % G]], None, N, t0,
                                          mb["outer_lr"], mb["outer_beta"]), iters)
        res[label] = dict(ms=ms, bytes_per_param=bpp, GBps=P * bpp / ms / 1e6)
    for g in mb["replicas"]:
        bpp = 8 * g + 24 + 10 * g
        ms = timed(lambda i: A.k_dn_group(theta, m, delta, starts[:g], works[:g], lps[:g], g, 0, mb["outer_lr"],
                                          mb["outer_beta"], 0.0, restart=True), max(iters // 4, 5))
        res[f"dn_group_G{g}_N{g}_restart"] = dict(ms=ms, bytes_per_param=bpp, GBps=P * bpp / ms / 1e6)
    grad, am, av = rnd(1e-3), rnd(1e-3), rnd(1e-6).abs()
    step = [0]

    def adam(i):
        step[0] += 1
        A.k_adamw(works[i % G], grad, am, av, lps[i % G], P - 4096, step[0], 1e-3)
    ms = timed(adam, iters)
    res["adamw_fp32grad_bf16copy"] = dict(ms=ms, bytes_per_param=30, GBps=P * 30 / ms / 1e6)
    key = "dn_event_nonboundary_N4"
    out = dict(metric="DN/AdamW HBM GB/s", value=res[key]["GBps"], unit="GB/s", n_gpus=1, steps=iters, warmup=2,
               ms_per_step=res[key]["ms"], higher_is_better=True, scaling="weak", vs_baseline=None, dtype="f32",
               data="synthetic", config=dict(workload=f"outer_microbench: {P} fp32 parameters, 16 replicas resident, "
                                                      "value = one non-boundary Delayed-Nesterov event (N=4, c=0)", results=res),
               roofline=dict(bound="hbm", achieved=res[key]["GBps"], peak=PEAK_HBM_GBS, unit="GB/s",
                             frac=res[key]["GBps"] / PEAK_HBM_GBS,
                             # FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 of this launch (profiles/outer_microbench_dn_adamw.md)
                             traffic=(2343894 + 1171876) * 1024.0, kernel="dn_group_kernel<4>"),
               cpu_baseline=None if args.no_cpu_baseline else cpu_baseline_outer(mb))
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="lm20m")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--streams", type=int, default=0, help="HIP streams the workers share (worker i on stream i mod n); 0 = min(k, 4): the box gives a process 4 hardware queues")
    ap.add_argument("--gemm-tile", default="", help="tuning: force the MFMA GEMM tile, e.g. 256x128x1 (tile M x tile N x LDS buffers)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the simulated workers are replicas on HIP streams of "
              "a single MI355X); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.workload == "outer_microbench":
        return outer_microbench(args)

    import numpy as np
    import torch
    import als_inputs as I
    import paper_2401_09135_amd as A

    w = I.workload(args.workload)
    if args.gemm_tile:
        A.set_gemm_tile(*[int(x) for x in args.gemm_tile.split("x")])
    k, N = w["k"], w["N"]
    n_rounds = args.warmup + args.steps
    n_events = n_rounds * N
    steps, ev_w, ev_t, ev_g = A.dylu_schedule(w["speeds"], w["H"], w["tau_grace"], n_events)
    cfg = A.Config.from_workload(w, max_local_steps=int(steps.max()))
    # parameter layout from the library itself; values N(0, 0.02), gains 1
    P, Pd = A.param_count(cfg), A.param_count_decayed(cfg)
    theta0 = I.theta0([("decayed", (Pd,), "matrix"), ("gains", (P - Pd,), "gain")], w["seed"])
    ctx = A.Context(cfg, theta0, n_streams=args.streams or min(k, 4))

    # how many local rounds each worker starts: the first one plus one per sync event of its own
    rounds = [1 + int((ev_w == i).sum()) for i in range(k)]
    toks = []
    for i in range(k):
        st = I.TokenStream(w["seed"], i, w["B"], w["S"], w["V"])
        toks.append([torch.from_numpy(st.take(int(steps[i]))).to(ctx.device) for _ in range(rounds[i])])
    nxt = [0] * k

    def train(i):
        ctx.worker_local_steps(i, toks[i][nxt[i]], w["lr"])
        nxt[i] += 1

    def run_events(e0, e1):
        tokens = 0
        e = e0
        while e < e1:
            j = e
            while j < e1 - 1 and not ev_g[j]:
                j += 1
            group = [int(x) for x in ev_w[e:j + 1]]
            ctx.outer_apply_dn(group, restart=True)
            for i in group:
                tokens += int(steps[i]) * w["B"] * w["S"]
                train(i)
            e = j + 1
        return tokens

    for i in range(k):
        train(i)
    run_events(0, args.warmup * N)
    ctx.sync()
    torch.cuda.synchronize()
    # HIP events around every 16th MFMA GEMM launch of the timed region, on the launching stream
    # (timing every launch costs 5 % of the throughput being measured)
    A.prof_enable(16)
    t0 = time.perf_counter()
    tokens = run_events(args.warmup * N, n_events)
    ctx.sync()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    A.prof_enable(False)
    prof_overlapped = sorted(A.prof_collect(), key=lambda r: -r[2])
    # Kernel quality is measured right after the timed region with ONE worker stepping alone (two
    # local steps): in the timed region four workers' kernels share the chip, so a launch's
    # begin-to-end time there includes the time it spends waiting for CUs held by other streams.
    iso_tok = torch.from_numpy(I.TokenStream(w["seed"], 1000, w["B"], w["S"], w["V"]).take(2)).to(ctx.device)
    A.prof_enable(True)
    ctx.worker_local_steps(0, iso_tok, w["lr"])
    ctx.sync()
    A.prof_enable(False)
    prof = sorted(A.prof_collect(), key=lambda r: -r[2])

    tok_s = tokens / dt
    tflops = tok_s * flops_per_token(w) / 1e12
    out = dict(metric="simulated-worker training tokens/s/GPU", value=tok_s, unit="tokens/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=1e3 * dt / max(args.steps, 1),
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16" if w["dtype"] == "bf16" else "f32",
               data="synthetic",
               config=dict(workload=f"{args.workload}: L{w['L']} d{w['d']} h{w['h']} ff{w['ff']} V{w['V']} S{w['S']} "
                                    f"B{w['B']}/worker, k={k} workers speeds {np.round(w['speeds'], 3).tolist()}, "
                                    f"DyLU H={w['H']} -> {steps.tolist()}, DN N={N} beta={w['outer_beta']} "
                                    f"eps={w['outer_lr']}, step = one outer round of N sync events",
                           tokens_per_step=tokens // max(args.steps, 1),
                           model_tflops=tflops, mfma_frac_whole_path=tflops / PEAK_BF16_TFLOPS),
               roofline=None, cpu_baseline=None)
    if prof:
        # dominant kernel = the GEMM instantiation with the largest summed duration
        name, launches, ms, fl = prof[0]
        achieved = fl / (ms * 1e-3) / 1e12
        out["roofline"] = dict(bound="mfma", achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                               frac=achieved / PEAK_BF16_TFLOPS,
                               traffic=MEASURED_TRAFFIC_BYTES.get(args.workload, {}).get(name), kernel=name, launches=launches,
                               avg_us=1e3 * ms / launches, flops_per_launch=fl / launches,
                               how="HIP events around every launch of this kernel while one worker steps alone "
                                   "right after the timed region (same shapes, same stream)",
                               all_gemm_kernels=[dict(kernel=n, launches=l, avg_us=1e3 * m / l,
                                                      tflops=f / (m * 1e-3) / 1e12) for n, l, m, f in prof],
                               timed_region_overlapped=[dict(kernel=n, launches=l, avg_us=1e3 * m / l,
                                                             tflops=f / (m * 1e-3) / 1e12)
                                                        for n, l, m, f in prof_overlapped])
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    ctx.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
