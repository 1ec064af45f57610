"""Benchmark of the asynchronous Local-SGD hot path on one MI355X.

Headline (default run): the 150M-class workload (benchmark configs[3], the largest configuration
that runs on one GPU).  A "step" is one outer round of the paper's asynchronous schedule: N = 4 sync
events (pseudo-gradient + Delayed Nesterov + restart) together with the local rounds of the four
simulated workers (DyLU step counts, each step = forward + backward + AdamW on 16 x 1024 tokens),
which run on their own HIP streams.  Tokens are synthetic Zipf(1.1) draws, resident in HBM before the
clock starts.  The default run then also measures the 20M-class workload (configs[1]), the same model
with 16 workers (configs[4], with the outer-step overhead fraction) and the outer-step
microbenchmark (configs[2]) and reports them under config.other_workloads.  Prints ONE JSON line.

  python bench.py                                  the default run described above
  python bench.py --workload lm20m                 one workload only
  python bench.py --workload outer_microbench      configs[2] only
  python bench.py --workload gemm_microbench [--tiles 256x128x1,128x128x2]
                                                   the MFMA GEMM on the step's shapes, one kernel at a
                                                   time on one stream (the program behind the counter
                                                   runs in profiles/)
  python bench.py --workload dw_grouped_sweep      the grouped weight-gradient launch on equal products
                                                   of growing operand footprint
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
HEADLINE = "lm150m"
CONFIG_FLAGS = 0            # als_config.flags of the timed contexts (--config-flags; 2 = one weight-gradient product per matrix)
# Bytes moved behind the L2s per launch of the dominant GEMM kernel of a workload, measured with
# rocprofv3 --pmc FETCH_SIZE (x 2.0) and WRITE_SIZE (x 1.0) on the same shapes, one kernel at a time
# (profiles/gemm_mfma_microbench.md gives the commands, the calibration of the two factors and the
# comparison with the algorithmic bytes), averaged over the launch mix of a worker step.  Counters
# cannot be collected from inside this process, so the figure is carried here, keyed by workload and
# kernel, next to the algorithmic bytes of the same launches (operands once + split-K partials
# written); a kernel without an entry reports null, never another kernel's figure.
MEASURED_TRAFFIC_BYTES = {"lm20m": {"gemm_pp_kernel<0, 1, STORE, float, false>": 127.3e6,
                                    "gemm_pp_dw_grouped_kernel": 1980.1e6,
                                    "gemm_pp_kernel<1, 0, STORE, float, true>": 135.5e6},
                          "lm150m": {"gemm_pp_dw_grouped_kernel": 10422.5e6,
                                     "gemm_pp_kernel<1, 0, STORE, float, true>": 211.9e6}}
ALGORITHMIC_TRAFFIC_BYTES = {"lm20m": {"gemm_pp_kernel<0, 1, STORE, float, false>": 110.7e6,
                                       "gemm_pp_dw_grouped_kernel": 1753.1e6,
                                       "gemm_pp_kernel<1, 0, STORE, float, true>": 133.9e6},
                             "lm150m": {"gemm_pp_dw_grouped_kernel": 6166.8e6,
                                        "gemm_pp_kernel<1, 0, STORE, float, true>": 168.0e6}}


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


def cpu_baseline(w):
    """The oracle as it stands, timed on the host: local steps (forward, backward, AdamW) of
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


def outer_microbench(steps):
    """Benchmark configs[2]: pseudo-gradient + Delayed Nesterov (single events, the grouped pass with
    fused restart) and fused AdamW on a 150M-element fp32 vector; achieved HBM GB/s from the
    algorithmic bytes per parameter (DN: 24 non-boundary, 32 boundary, grouped G events with
    restart 8G + 24 + 10G; AdamW: 30 with fp32 gradient and bf16 copy).  Returns the result table."""
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

    iters = max(steps, 20)
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
    res["_iters"] = iters
    del theta, m, delta, starts, works, lps, grad, am, av
    torch.cuda.empty_cache()
    return res


def outer_microbench_line(args):
    import als_inputs as I
    mb = I.OUTER_MICROBENCH
    res = outer_microbench(args.steps)
    iters = res.pop("_iters")
    # configs[2] is the fused pass over 4-16 replicas: the reported value is the grouped pass over 4
    # workers with the restart fused in (the single events and the larger groups are in results)
    key = "dn_group_G4_N4_restart"
    out = dict(metric="DN/AdamW HBM GB/s", value=res[key]["GBps"], unit="GB/s", n_gpus=1, steps=iters, warmup=2,
               ms_per_step=res[key]["ms"], higher_is_better=True, scaling="weak", vs_baseline=None, dtype="f32",
               data="synthetic", config=dict(workload=f"outer_microbench: {mb['P']} fp32 parameters, 16 replicas resident, "
                                                      "value = one fused pass of 4 Delayed-Nesterov events (N=4, c=0) "
                                                      "with the 4 workers' restart", results=res),
               roofline=dict(bound="hbm", achieved=res[key]["GBps"], peak=PEAK_HBM_GBS, unit="GB/s",
                             frac=res[key]["GBps"] / PEAK_HBM_GBS,
                             # FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 of the pass's two launches
                             # (profiles/outer_microbench_dn_adamw.md): the algorithmic 96 bytes per
                             # parameter plus the restart pass's second read of theta
                             traffic=(6445674 + 1757813 + 585971 + 5859375) * 1024.0,
                             kernel="dn_group_kernel<2> + restart_group_kernel"),
               cpu_baseline=None if args.no_cpu_baseline else cpu_baseline_outer(mb))
    print(json.dumps(out))


# name, M, N, K, a_layout, b_layout, epilogue (-1: plain store to fp32, 0: store bf16, 1 residual, 2 GELU, 3 x derivative)
def gemm_shapes(w):
    T, d, ff, V = w["B"] * w["S"], w["d"], w["ff"], w["V"]
    a = w["h"] * w["dh"] if w.get("dh") else d
    return [("qkv", T, 3 * a, d, 0, 0, 0), ("wo+res", T, d, a, 0, 0, 1), ("ffn1+gelu", T, ff, d, 0, 0, 2),
            ("ffn2+res", T, d, ff, 0, 0, 1), ("head bf16", T, V, d, 0, 0, 0),
            ("dffn2*gp", T, ff, d, 0, 1, 3), ("dffn1 f32", T, d, ff, 0, 1, -1), ("dqkv f32", T, d, 3 * a, 0, 1, -1),
            ("do bf16", T, a, d, 0, 1, 0), ("dhead f32", T, d, V, 0, 1, -1),
            ("dw ffn1", d, ff, T, 1, 0, 0), ("dw ffn2", ff, d, T, 1, 0, 0), ("dw qkv", d, 3 * a, T, 1, 0, 0),
            ("dw wo", a, d, T, 1, 0, 0), ("dw head", d, V, T, 1, 0, 0)]


def gemm_microbench(args):
    """The MFMA GEMM kernel on the GEMM shapes of a worker step (default: the headline workload), each
    with the epilogue the step uses, through the C ABI (als_k_gemm_ex), one kernel at a time on one
    stream; --tiles forces tile variants (tile M x tile N x LDS buffers) next to the automatic choice."""
    import torch
    import als_inputs as I
    import paper_2401_09135_amd as A
    dev = "cuda:0"
    names = [args.shapes_of] if args.shapes_of else [HEADLINE, "lm20m"]
    # calibration for HBM counter runs: three plain device copies of 2^26 floats (256 MiB read and
    # 256 MiB written each) appear in a rocprofv3 --pmc run as launches of known traffic
    cal_src = torch.randn(1 << 26, device=dev)
    cal_dst = torch.empty_like(cal_src)
    for _ in range(3):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_src, cal_dst
    ws = torch.empty(64 << 20, dtype=torch.uint8, device=dev)     # split-K scratch
    tiles = [(0, 0, 0)] + [tuple(int(x) for x in t.split("x")) for t in args.tiles.split(",") if t]
    rows = []
    for wname in names:
        shapes = gemm_shapes(I.workload(wname)) + ([("square 8192", 8192, 8192, 8192, 0, 1, 0)] if wname == names[-1] else [])
        for name, M, N, K, al, bl, epi in shapes:
            a = torch.randn((M, K) if al == 0 else (K, M), device=dev).to(torch.bfloat16)
            b = torch.randn((K, N) if bl == 0 else (N, K), device=dev).to(torch.bfloat16)
            e = max(epi, 0)
            out_f32 = e == 1 or al == 1 or epi == -1
            c = torch.empty(M, N, dtype=torch.float32 if out_f32 else torch.bfloat16, device=dev)
            R = torch.randn(M, N, device=dev) if e == 1 else None
            C2 = torch.empty(M, N, dtype=torch.bfloat16, device=dev) if e == 2 else None
            U = torch.randn(M, N, device=dev).to(torch.bfloat16) if e == 3 else None
            for tile in tiles:
                A.set_gemm_tile(*tile)
                f = lambda: A.k_gemm_ex(a, b, c, M, N, K, al, bl, True, e, R, C2, U, ws if al == 1 else None)
                try:
                    for _ in range(10):   # first launches on fresh buffers run up to 10 % slower
                        f()
                    torch.cuda.synchronize()
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record()
                    for _ in range(args.steps):
                        f()
                    e1.record()
                    torch.cuda.synchronize()
                    ms = e0.elapsed_time(e1) / args.steps
                    rows.append(dict(workload=wname, product=name, M=M, N=N, K=K, tile="auto" if not tile[0] else "x".join(map(str, tile)),
                                     us=ms * 1e3, tflops=2.0 * M * N * K / ms / 1e9))
                    print(f"{wname:8s} {name:12s} M{M:<6d} N{N:<6d} K{K:<6d} tile={rows[-1]['tile']:10s}: {ms * 1e3:8.1f} us "
                          f"{rows[-1]['tflops']:6.0f} TFLOP/s", file=sys.stderr, flush=True)
                except A.AlsError as ex:
                    print(f"{wname:8s} {name:12s} tile={tile}: not supported ({str(ex)[:60]})", file=sys.stderr, flush=True)
                finally:
                    A.set_gemm_tile(0, 0, 0)
            del a, b, c, R, C2, U
        # all layers' weight gradients as the backward pass runs them: one grouped launch
        w = I.workload(wname)
        T, d, ff = w["B"] * w["S"], w["d"], w["ff"]
        a_w = w["h"] * w["dh"] if w.get("dh") else d
        layer = [(d, 3 * a_w), (a_w, d), (d, ff), (ff, d)]
        if all(m % 128 == 0 and n % 128 == 0 for m, n in layer):
            Xs = [torch.randn(T, m, device=dev).to(torch.bfloat16) for m, _ in layer * w["L"]]
            dYs = [torch.randn(T, n, device=dev).to(torch.bfloat16) for _, n in layer * w["L"]]
            Cs = [torch.empty(m, n, device=dev) for m, n in layer * w["L"]]
            gws = torch.empty(A.k_gemm_dw_grouped_ws_bytes([m for m, _ in layer * w["L"]], [n for _, n in layer * w["L"]]),
                              dtype=torch.uint8, device=dev)
            f = lambda: A.k_gemm_dw_grouped(Xs, dYs, Cs, T, gws)
            for _ in range(3):
                f()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(max(args.steps // 4, 3)):
                f()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / max(args.steps // 4, 3)
            fl = sum(2.0 * m * n * T for m, n in layer) * w["L"]
            rows.append(dict(workload=wname, product=f"dw grouped ({4 * w['L']} products)", M=0, N=0, K=T, tile="auto", us=ms * 1e3, tflops=fl / ms / 1e9))
            print(f"{wname:8s} dw grouped, {4 * w['L']} products, one launch: {ms * 1e3:8.1f} us {rows[-1]['tflops']:6.0f} TFLOP/s", file=sys.stderr, flush=True)
            del Xs, dYs, Cs, gws
    auto = [r for r in rows if r["tile"] == "auto" and r["product"] != "square 8192"]
    best = max(auto, key=lambda r: r["tflops"])
    print(json.dumps(dict(metric="MFMA GEMM TFLOP/s on the worker step's products", value=best["tflops"], unit="TFLOP/s",
                          n_gpus=1, steps=args.steps, warmup=10, ms_per_step=best["us"] / 1e3, higher_is_better=True,
                          scaling="weak", vs_baseline=None, dtype="bf16", data="synthetic",
                          config=dict(workload="gemm_microbench: " + ", ".join(names), results=rows),
                          roofline=dict(bound="mfma", achieved=best["tflops"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                                        frac=best["tflops"] / PEAK_BF16_TFLOPS, traffic=None,
                                        kernel=f"{best['workload']} {best['product']}"), cpu_baseline=None)))


def dw_grouped_sweep(args):
    """The grouped weight-gradient launch (als_k_gemm_dw_grouped) on n equal products m x m over
    K = 16384 tokens, n m^2 fixed: how its rate depends on the operand bytes that have to come from
    beyond the L2s.  Each size runs with every product on operands of its own, and with the products
    sharing 1, 2 or 16 operand pairs (pair p mod c), which keeps the L2 behaviour of the distinct case
    for c >= 2 while the operands fit (or do not fit) the 256 MB last-level cache."""
    import torch
    import paper_2401_09135_amd as A
    dev, T = "cuda:0", 16384
    rows = []
    for n, m in ((1024, 256), (256, 512), (64, 1024), (16, 2048), (1, 8192)):
        for pairs in ([n, 16, 2, 1] if m in (512, 1024) else [n]):
            X0 = [(torch.randn(T, m, device=dev) * 0.5).to(torch.bfloat16) for _ in range(pairs)]
            Y0 = [(torch.randn(T, m, device=dev) * 0.5).to(torch.bfloat16) for _ in range(pairs)]
            Xs, Ys = [X0[p % pairs] for p in range(n)], [Y0[p % pairs] for p in range(n)]
            Cs = [torch.empty(m, m, device=dev) for _ in range(n)]
            ws = torch.empty(A.k_gemm_dw_grouped_ws_bytes([m] * n, [m] * n), dtype=torch.uint8, device=dev)
            best = 1e30
            for _ in range(3):
                A.k_gemm_dw_grouped(Xs, Ys, Cs, T, ws)
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(args.steps):
                    A.k_gemm_dw_grouped(Xs, Ys, Cs, T, ws)
                e1.record()
                torch.cuda.synchronize()
                best = min(best, e0.elapsed_time(e1) / args.steps)
            rows.append(dict(products=n, m=m, operand_pairs=pairs, us=best * 1e3, tflops=2.0 * n * m * m * T / best / 1e9,
                             unique_operand_TBps=4.0 * pairs * m * T / best / 1e9))
            print(f"{n:5d} x {m:4d}^2, {pairs:4d} operand pair(s) ({4e-6 * pairs * m * T:7.0f} MB): {best * 1e3:7.0f} us "
                  f"{rows[-1]['tflops']:6.0f} TFLOP/s, unique operand bytes at {rows[-1]['unique_operand_TBps']:.2f} TB/s",
                  file=sys.stderr, flush=True)
            del X0, Y0, Xs, Ys, Cs, ws
    best = max(rows, key=lambda r: r["tflops"])
    print(json.dumps(dict(metric="grouped weight-gradient launch, TFLOP/s", value=best["tflops"], unit="TFLOP/s", n_gpus=1,
                          steps=args.steps, warmup=1, ms_per_step=best["us"] / 1e3, higher_is_better=True, scaling="weak",
                          vs_baseline=None, dtype="bf16", data="synthetic",
                          config=dict(workload="dw_grouped_sweep: n products m x m over K = 16384", results=rows),
                          roofline=dict(bound="mfma", achieved=best["tflops"], peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                                        frac=best["tflops"] / PEAK_BF16_TFLOPS, traffic=None, kernel="gemm_pp_dw_grouped_kernel"),
                          cpu_baseline=None)))


def run_lm(name, steps_timed, warmup, n_streams, isolated_profile=True):
    """Runs warmup + steps_timed outer rounds of one language-model workload and returns the measured
    figures.  Groups of events (ties, grace windows) are applied as the library's schedule marks them
    (a group restarts only when its last event carries the group-end flag), exactly as the driver
    loop the parity tests use; the timed region starts at a group end."""
    import numpy as np
    import torch
    import als_inputs as I
    import paper_2401_09135_amd as A

    w = I.workload(name)
    k, N = w["k"], w["N"]
    n_events = (warmup + steps_timed) * N
    steps, ev_w, ev_t, ev_g = A.dylu_schedule(w["speeds"], w["H"], w["tau_grace"], n_events)
    cfg = A.Config.from_workload(w, flags=CONFIG_FLAGS, max_local_steps=int(steps.max()))
    # parameter layout from the library itself; values N(0, 0.02), gains 1
    P, Pd = A.param_count(cfg), A.param_count_decayed(cfg)
    theta0 = I.theta0([("decayed", (Pd,), "matrix"), ("gains", (P - Pd,), "gain")], w["seed"])
    ctx = A.Context(cfg, theta0, n_streams=n_streams or min(k, 4))

    # the schedule's groups: (first event, last event, restarts?)
    groups, e = [], 0
    while e < n_events:
        j = e
        while j < n_events - 1 and not ev_g[j]:
            j += 1
        groups.append((e, j, bool(ev_g[j])))
        e = j + 1
    # the timed region starts with the first group that begins at or after event warmup * N
    first_timed = next(gi for gi, g in enumerate(groups) if g[0] >= warmup * N) if steps_timed else len(groups)

    # how many local rounds each worker starts: the first one plus one per restart
    rounds = [1] * k
    for (a, b, complete) in groups:
        if complete:
            for i in ev_w[a:b + 1]:
                rounds[int(i)] += 1
    toks = []
    for i in range(k):
        st = I.TokenStream(w["seed"], i, w["B"], w["S"], w["V"])
        toks.append([torch.from_numpy(st.take(int(steps[i]))).to(ctx.device) for _ in range(rounds[i])])
    nxt = [0] * k

    def train(i):
        ctx.worker_local_steps(i, toks[i][nxt[i]], w["lr"])
        nxt[i] += 1

    def run_groups(g0, g1):
        tokens = events = 0
        for (a, b, complete) in groups[g0:g1]:
            group = [int(x) for x in ev_w[a:b + 1]]
            ctx.outer_apply_dn(group, restart=complete)
            events += len(group)
            if complete:
                for i in group:
                    tokens += int(steps[i]) * w["B"] * w["S"]
                    train(i)
        return tokens, events

    for i in range(k):
        train(i)
    run_groups(0, first_timed)
    ctx.sync()
    torch.cuda.synchronize()
    # HIP events around every 16th MFMA GEMM launch of the timed region, on the launching stream
    # (timing every launch costs 5 % of the throughput being measured)
    A.prof_enable(16)
    t0 = time.perf_counter()
    tokens, events = run_groups(first_timed, len(groups))
    ctx.sync()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    A.prof_enable(False)
    prof_overlapped = sorted(A.prof_collect(), key=lambda r: -r[2])

    # Outer-step cost (pseudo-gradient + Delayed Nesterov + restart copies): every distinct group size
    # of the timed region applied alone on an idle GPU, host-timed between two synchronisations
    # (the replicas hold the server's parameters, so the pseudo-gradients are zero: same bytes moved).
    sizes = {}
    for (a, b, complete) in groups[first_timed:]:
        sizes[(b - a + 1, complete)] = sizes.get((b - a + 1, complete), 0) + 1
    outer_s = 0.0
    for (gsz, complete), count in sizes.items():
        grp = list(range(gsz))
        ctx.outer_apply_dn(grp, restart=complete)
        ctx.sync()
        ts = time.perf_counter()
        for _ in range(3):
            ctx.outer_apply_dn(grp, restart=complete)
        ctx.sync()
        outer_s += count * (time.perf_counter() - ts) / 3

    # Kernel quality is measured right after the timed region with ONE worker stepping alone (two
    # local steps): in the timed region the workers' kernels share the chip, so a launch's
    # begin-to-end time there includes the time it spends waiting for CUs held by other streams.
    prof = []
    if isolated_profile:
        iso_tok = torch.from_numpy(I.TokenStream(w["seed"], 1000, w["B"], w["S"], w["V"]).take(2)).to(ctx.device)
        A.prof_enable(True)
        ctx.worker_local_steps(0, iso_tok, w["lr"])
        ctx.sync()
        A.prof_enable(False)
        prof = sorted(A.prof_collect(), key=lambda r: -r[2])
    ctx.close()
    del ctx, toks
    torch.cuda.empty_cache()

    rounds_timed = events / N if N else 0.0
    tok_s = tokens / dt if dt > 0 else 0.0
    tflops = tok_s * flops_per_token(w) / 1e12
    res = dict(workload=name,
               describe=f"{name}: L{w['L']} d{w['d']} h{w['h']} ff{w['ff']} V{w['V']} S{w['S']} B{w['B']}/worker, k={k} workers "
                        f"speeds {np.round(w['speeds'], 3).tolist()}, DyLU H={w['H']} -> {steps.tolist()}, DN N={N} "
                        f"beta={w['outer_beta']} eps={w['outer_lr']}, step = one outer round of N sync events",
               tokens_per_s=tok_s, seconds=dt, sync_events_timed=events, outer_rounds_timed=rounds_timed,
               ms_per_outer_round=1e3 * dt / rounds_timed if rounds_timed else None,
               tokens_per_outer_round=tokens / rounds_timed if rounds_timed else None,
               model_tflops=tflops, mfma_frac_whole_path=tflops / PEAK_BF16_TFLOPS,
               outer_step_seconds_isolated=outer_s, outer_step_overhead_fraction=outer_s / dt if dt > 0 else None,
               w=w)
    if prof:
        # dominant kernel = the GEMM instantiation with the largest summed duration
        kname, launches, ms, fl = prof[0]
        achieved = fl / (ms * 1e-3) / 1e12
        res["roofline"] = dict(bound="mfma", achieved=achieved, peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                               frac=achieved / PEAK_BF16_TFLOPS,
                               traffic=MEASURED_TRAFFIC_BYTES.get(name, {}).get(kname),
                               traffic_algorithmic=ALGORITHMIC_TRAFFIC_BYTES.get(name, {}).get(kname), kernel=kname, launches=launches,
                               avg_us=1e3 * ms / launches, flops_per_launch=fl / launches,
                               how="HIP events around every launch of this kernel while one worker steps alone "
                                   "right after the timed region (same shapes, same stream)",
                               all_gemm_kernels=[dict(kernel=n, launches=l, avg_us=1e3 * m / l,
                                                      tflops=f / (m * 1e-3) / 1e12) for n, l, m, f in prof],
                               gemm_tflops_all_kernels=sum(f for _, _, _, f in prof) / (sum(m for _, _, m, _ in prof) * 1e-3) / 1e12,
                               timed_region_overlapped=[dict(kernel=n, launches=l, avg_us=1e3 * m / l,
                                                             tflops=f / (m * 1e-3) / 1e12)
                                                        for n, l, m, f in prof_overlapped])
    return res


def achieved_ceilings():
    """What this machine gives plain kernels, so that the fractions of the published peaks can be read:
    a device-to-device copy of 1 GiB (read + written bytes per second) and the library's own GEMM
    on an 8192-cube with every operand resident in the last-level cache."""
    import torch
    import paper_2401_09135_amd as A
    dev = "cuda:0"
    src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
    dst = torch.empty_like(src)

    def timed(fn, n):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n
    ms_copy = timed(lambda: dst.copy_(src), 20)
    del src, dst
    n = 8192
    a = torch.randn(n, n, device=dev).to(torch.bfloat16)
    b = torch.randn(n, n, device=dev).to(torch.bfloat16)
    c = torch.empty(n, n, dtype=torch.bfloat16, device=dev)
    ms_gemm = timed(lambda: A.k_gemm_ex(a, b, c, n, n, n, 0, 1, True, 0, None, None, None, None), 20)
    return dict(copy_GBps=2.0 * 4 * (1 << 28) / ms_copy / 1e6, copy_frac_of_hbm_peak=2.0 * 4 * (1 << 28) / ms_copy / 1e6 / PEAK_HBM_GBS,
                gemm_8192_cube_tflops=2.0 * n ** 3 / ms_gemm / 1e9, gemm_8192_cube_frac_of_peak=2.0 * n ** 3 / ms_gemm / 1e9 / PEAK_BF16_TFLOPS,
                note="device copy of 1 GiB (torch copy_) and als_k_gemm_ex on an 8192-cube (bf16, A row-major, B column-major), 20 launches each after 10 untimed, "
                     "taken right after the timed workloads, in the power state they leave the chip in")


def _brief(r):
    keep = ("describe", "tokens_per_s", "ms_per_outer_round", "outer_rounds_timed", "model_tflops",
            "mfma_frac_whole_path", "outer_step_overhead_fraction", "outer_step_seconds_isolated")
    out = {k: r[k] for k in keep}
    if "roofline" in r:
        out["dominant_gemm"] = {k: r["roofline"][k] for k in ("kernel", "achieved", "frac", "avg_us")}
        out["gemm_tflops_all_kernels"] = r["roofline"]["gemm_tflops_all_kernels"]
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=8)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="", help="one workload only (lm150m, lm20m, lm20m_k16, paper150m_b128, "
                                                   "outer_microbench, gemm_microbench, dw_grouped_sweep); default: the headline "
                                                   f"workload ({HEADLINE}) followed by short runs of the others")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="default run: skip the other workloads")
    ap.add_argument("--streams", type=int, default=0, help="HIP streams the workers share (worker i on stream i mod n); 0 = min(k, 4): the box gives a process 4 hardware queues")
    ap.add_argument("--config-flags", type=int, default=0, help="tuning: als_config.flags of the timed contexts (bit 1: one weight-gradient product per matrix instead of the grouped launch)")
    ap.add_argument("--gemm-tile", default="", help="tuning: force the MFMA GEMM tile, e.g. 256x128x1 (tile M x tile N x LDS buffers)")
    ap.add_argument("--tiles", default="", help="gemm_microbench: comma-separated tile variants to time next to the automatic choice")
    ap.add_argument("--shapes-of", default="", help="gemm_microbench: the workload whose GEMM shapes are timed")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the simulated workers are replicas on HIP streams of "
              "a single MI355X); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    if args.workload == "outer_microbench":
        return outer_microbench_line(args)
    if args.workload == "gemm_microbench":
        return gemm_microbench(args)
    if args.workload == "dw_grouped_sweep":
        return dw_grouped_sweep(args)

    import paper_2401_09135_amd as A
    global CONFIG_FLAGS
    CONFIG_FLAGS = args.config_flags
    if args.gemm_tile:
        A.set_gemm_tile(*[int(x) for x in args.gemm_tile.split("x")])
    name = args.workload or HEADLINE
    r = run_lm(name, args.steps, args.warmup, args.streams)
    w = r["w"]
    out = dict(metric="simulated-worker training tokens/s/GPU", value=r["tokens_per_s"], unit="tokens/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=r["ms_per_outer_round"],
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="bf16" if w["dtype"] == "bf16" else "f32",
               data="synthetic",
               config=dict(workload=r["describe"], tokens_per_step=r["tokens_per_outer_round"],
                           sync_events_timed=r["sync_events_timed"], model_tflops=r["model_tflops"],
                           mfma_frac_whole_path=r["mfma_frac_whole_path"],
                           outer_step_overhead_fraction=r["outer_step_overhead_fraction"]),
               roofline=r.get("roofline"), cpu_baseline=None)
    if not args.workload and not args.no_others:
        # the other BASELINE configurations, short runs, reported beside the headline
        others = {}
        for oname, st, wu in (("lm20m", 4, 1), ("lm20m_k16", 2, 1)):
            others[oname] = _brief(run_lm(oname, st, wu, args.streams))
        mb = outer_microbench(20)
        mb.pop("_iters")
        others["outer_microbench"] = {k: dict(GBps=v["GBps"], frac_of_hbm_peak=v["GBps"] / PEAK_HBM_GBS, ms=v["ms"],
                                              bytes_per_param=v["bytes_per_param"]) for k, v in mb.items()}
        out["config"]["other_workloads"] = others
        if out["roofline"] is not None:
            out["roofline"]["achieved_ceilings"] = achieved_ceilings()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
