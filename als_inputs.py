"""Seeded synthetic inputs and workload tables shared by the CPU oracle, the tests and the
benchmarks.

This module holds data recipes only: named workload shapes, token sampling, initial
parameter values, worker speeds.  It contains none of the method's arithmetic (no model,
no optimiser, no scheduler) and imports neither the oracle nor the HIP library, so both
sides can be fed exactly the same arrays.

Tokens are i.i.d. draws from a bounded Zipf law p(r) ~ r**-1.1 over ranks 1..V (token id
= rank - 1), sampled by inverse CDF; they stand in for the web-text corpus the paper trains
on, which cannot be shipped here.
"""
from __future__ import annotations

import numpy as np

# ---------------------------------------------------------------------------------------
# Workload tables (pure data).  Keys follow the paper's notation: L layers, d model width,
# h heads, ff FFN width, V vocabulary, S sequence length, B batch per worker, k workers,
# H the fastest worker's local step count (DyLU), N the Delayed-Nesterov buffer size.
# ---------------------------------------------------------------------------------------
_COMMON = dict(lr=1e-3, wd=0.1, beta1=0.9, beta2=0.999, adam_eps=1e-8, norm_eps=1e-5,
               outer_lr=0.7, outer_beta=0.9, dn_c=0.0, tau_grace=0.0, zipf_a=1.1, seed=0)

WORKLOADS = {
    # benchmark configs[0]: fp32 correctness case, 3 outer rounds = 12 sync events.
    "tiny": dict(_COMMON, L=2, d=64, h=2, ff=256, V=256, S=32, B=8, dtype="f32", k=4,
                 speeds=[1.0, 1.5, 2.0, 3.0], H=5, N=4, n_events=12),
    # benchmark configs[1]: the 20M-class LM the headline metric is quoted on.
    "lm20m": dict(_COMMON, L=6, d=512, h=8, ff=2048, V=8192, S=512, B=32, dtype="bf16", k=4,
                  speeds=[1.0, 1.2, 1.6, 2.4], H=50, N=4, n_events=4),
    # benchmark configs[3]: 150M-class LM; speeds drawn U[1,3] from the seed.
    "lm150m": dict(_COMMON, L=12, d=896, h=14, ff=3584, V=32000, S=1024, B=16, dtype="bf16",
                   k=4, speeds=("uniform", 1.0, 3.0), H=50, N=4, n_events=4),
    # benchmark configs[4]: 16 simulated workers sharing the GPU; speeds U[1,4].
    "lm20m_k16": dict(_COMMON, L=6, d=512, h=8, ff=2048, V=8192, S=512, B=32, dtype="bf16",
                      k=16, speeds=("uniform", 1.0, 4.0), H=50, N=16, n_events=16),
    # Reduced cases for parity tests (same architecture class, sizes the oracle finishes in
    # seconds, still several GEMM/attention tiles with ragged step counts).
    "mini_bf16": dict(_COMMON, L=2, d=256, h=4, ff=1024, V=1024, S=128, B=4, dtype="bf16",
                      k=4, speeds=[1.0, 1.2, 1.6, 2.4], H=10, N=4, n_events=4),
    # The paper's own model table (appendix, Model Configuration): 20M = 6 layers, hidden 256, 4
    # heads; 60M = 3 layers, hidden 896, 16 heads; 150M = 12 layers, hidden 896, 16 heads; K/V
    # size 64 (so the attention width of the two larger models is 1024, not 896), vocabulary
    # 32000, sequence 256.  FFN width 4 d (not printed).  Small per-worker batches for tests.
    "paper20m": dict(_COMMON, L=6, d=256, h=4, dh=64, ff=1024, V=32000, S=256, B=2, dtype="bf16",
                     k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    "paper60m": dict(_COMMON, L=3, d=896, h=16, dh=64, ff=3584, V=32000, S=256, B=2, dtype="bf16",
                     k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    "paper150m": dict(_COMMON, L=12, d=896, h=16, dh=64, ff=3584, V=32000, S=256, B=2, dtype="bf16",
                      k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    # the paper's 150M model at its own per-worker batch (128 sequences of 256): a bench workload
    "paper150m_b128": dict(_COMMON, L=12, d=896, h=16, dh=64, ff=3584, V=32000, S=256, B=128,
                           dtype="bf16", k=4, speeds=[1.0, 1.2, 1.6, 2.4], H=50, N=4, n_events=4),
    # layer normalisation (gain, no bias) instead of RMS normalisation, fp32 and bf16
    "tiny_ln": dict(_COMMON, L=2, d=64, h=2, ff=256, V=256, S=32, B=8, dtype="f32", k=4, norm="layer",
                    speeds=[1.0, 1.5, 2.0, 3.0], H=5, N=4, n_events=8),
    "mini_bf16_ln": dict(_COMMON, L=2, d=256, h=4, ff=1024, V=1024, S=128, B=4, dtype="bf16", norm="layer",
                         k=4, speeds=[1.0, 1.2, 1.6, 2.4], H=10, N=4, n_events=4),
    # bf16 mode on shapes no MFMA kernel accepts (T = 72, head width 32, V = 200): the generic
    # GEMM / attention kernels with bf16 operands
    "ragged_bf16": dict(_COMMON, L=2, d=64, h=2, ff=128, V=200, S=24, B=3, dtype="bf16",
                        k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=4),
    "wide_attn_f32": dict(_COMMON, L=2, d=64, h=4, dh=32, ff=128, V=200, S=24, B=3, dtype="f32",
                          k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=4),
    # the 150M-class architecture on one 1024-token sequence per step (d 896 = 7 x 128, 14 heads,
    # V 32000, S 1024): every kernel shape class of benchmark configs[3] at 1/16 of its batch
    "lm150m_b1": dict(_COMMON, L=12, d=896, h=14, ff=3584, V=32000, S=1024, B=1, dtype="bf16",
                      k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    # 16 heterogeneous workers (benchmark configs[4]'s scheduling shape) on the reduced model
    "mini_bf16_k16": dict(_COMMON, L=2, d=256, h=4, ff=1024, V=1024, S=128, B=2, dtype="bf16",
                          k=16, speeds=("uniform", 1.0, 4.0), H=6, N=16, n_events=16),
    # grace period > 0 and momentum activation c > 0 (the paper's ablation knobs), fp32 and bf16
    "tiny_grace_c": dict(_COMMON, L=2, d=64, h=2, ff=256, V=256, S=32, B=8, dtype="f32", k=4,
                         speeds=[1.0, 1.5, 2.0, 3.0], H=5, N=4, n_events=12, tau_grace=0.2, dn_c=0.1),
    "mini_bf16_grace_c": dict(_COMMON, L=2, d=256, h=4, ff=1024, V=1024, S=128, B=4, dtype="bf16",
                              k=4, speeds=[1.0, 1.2, 1.6, 2.4], H=10, N=4, n_events=8, tau_grace=0.5, dn_c=0.25),
    "mini_f32": dict(_COMMON, L=2, d=128, h=4, ff=384, V=320, S=48, B=3, dtype="f32",
                     k=3, speeds=[1.0, 2.0, 2.0], H=4, N=3, n_events=6),
    # edge shapes for parity tests: an odd vocabulary (no vector-width kernel applies to the logits),
    # the largest model width the norm kernels take, heads of 32 in bf16 mode (MFMA GEMMs with the
    # generic attention kernels), and sequences of a single position
    "edge_v_odd": dict(_COMMON, L=1, d=64, h=2, ff=128, V=201, S=16, B=2, dtype="bf16",
                       k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    "edge_d1024": dict(_COMMON, L=1, d=1024, h=16, ff=1024, V=256, S=128, B=1, dtype="bf16",
                       k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    "edge_dh32_bf16": dict(_COMMON, L=2, d=128, h=4, ff=256, V=256, S=128, B=2, dtype="bf16",
                           k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    # 20 workers of equal speed: every round ends in ONE tie group of 20 events, more than the 16 a
    # single pass of the fused outer kernel takes
    "tiny_k20": dict(_COMMON, L=1, d=64, h=2, ff=64, V=64, S=8, B=2, dtype="f32", k=20,
                     speeds=[1.0] * 20, H=2, N=20, n_events=40),
    # a vocabulary beyond the 32768 columns the register-resident cross-entropy kernel holds
    "edge_v_big": dict(_COMMON, L=1, d=64, h=2, ff=64, V=40000, S=8, B=2, dtype="bf16",
                       k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
    # a single worker (the asynchronous schedule degenerates to a chain of rounds), buffer N = 2
    "tiny_k1": dict(_COMMON, L=1, d=64, h=2, ff=64, V=64, S=8, B=2, dtype="f32", k=1,
                    speeds=[1.5], H=3, N=2, n_events=4),
    "edge_s1": dict(_COMMON, L=1, d=64, h=2, ff=64, V=64, S=1, B=4, dtype="f32",
                    k=2, speeds=[1.0, 2.0], H=2, N=2, n_events=2),
}

# benchmark configs[2]: the outer-step microbenchmark on a flat fp32 vector.
OUTER_MICROBENCH = dict(P=150_000_000, replicas=(4, 8, 16), N=(1, 4, 8), sigma=0.02,
                        drift_sigma=1e-3, outer_lr=0.7, outer_beta=0.9, seed=0)


def workload(name: str) -> dict:
    w = dict(WORKLOADS[name])
    w["name"] = name
    w["speeds"] = worker_speeds(w)
    return w


def worker_speeds(w: dict) -> np.ndarray:
    """Worker speeds in steps per second as an fp64 array (fixed list or seeded uniform)."""
    s = w["speeds"]
    if isinstance(s, tuple) and s[0] == "uniform":
        rng = np.random.default_rng([w["seed"], 0x5EED])
        return rng.uniform(s[1], s[2], size=w["k"]).astype(np.float64)
    return np.asarray(s, dtype=np.float64)


# ---------------------------------------------------------------------------------------
# Tokens
# ---------------------------------------------------------------------------------------
def zipf_cdf(V: int, a: float = 1.1) -> np.ndarray:
    p = np.arange(1, V + 1, dtype=np.float64) ** (-a)
    c = np.cumsum(p)
    return c / c[-1]


def zipf_tokens(rng: np.random.Generator, V: int, shape, a: float = 1.1) -> np.ndarray:
    """int32 token ids, i.i.d. bounded Zipf(a) over 0..V-1 by inverse CDF."""
    u = rng.random(size=shape)
    t = np.searchsorted(zipf_cdf(V, a), u, side="left")
    return np.minimum(t, V - 1).astype(np.int32)


class TokenStream:
    """Sequential batches for one worker: generator seeded by (seed, worker), each call to
    ``take(n)`` returns the next n batches as int32 [n, B, S+1]."""

    def __init__(self, seed: int, worker: int, B: int, S: int, V: int, a: float = 1.1):
        self.rng = np.random.default_rng([seed, worker])
        self.B, self.S, self.V, self.a = B, S, V, a

    def take(self, n: int) -> np.ndarray:
        return zipf_tokens(self.rng, self.V, (n, self.B, self.S + 1), self.a)


# ---------------------------------------------------------------------------------------
# Initial parameters.  ``layout`` is a list of (name, shape, kind) produced by whichever
# side asks (the oracle and the library each compute their own; tests check they agree);
# kind "matrix" -> N(0, sigma), kind "gain" -> 1.
# ---------------------------------------------------------------------------------------
def theta0(layout, seed: int = 0, sigma: float = 0.02) -> np.ndarray:
    rng = np.random.default_rng([seed, 0x7E7A])
    parts = []
    for _name, shape, kind in layout:
        n = int(np.prod(shape))
        if kind == "gain":
            parts.append(np.ones(n, dtype=np.float32))
        else:
            parts.append((rng.standard_normal(n) * sigma).astype(np.float32))
    return np.concatenate(parts)


def normal_vector(P: int, seed, sigma: float) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return (rng.standard_normal(P, dtype=np.float32) * np.float32(sigma)).astype(np.float32)
