"""GPU parity of the stand-alone kernels against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import als_inputs as I
import paper_2401_09135_amd as A
from oracle import lm
from oracle.optim import AdamW, DelayedNesterov

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


def _rel(a, b):
    return float(np.linalg.norm(a.astype(np.float64) - b.astype(np.float64)) / max(np.linalg.norm(b.astype(np.float64)), 1e-30))


@pytest.mark.parametrize("P", [0, 1, 5, 1000, 4 * 256 * 37 + 3, 1 << 20])
@pytest.mark.parametrize("N,c,G", [(1, 0.0, 1), (4, 0.0, 1), (4, 0.0, 4), (4, 0.1, 3), (3, 0.0, 7), (8, 0.05, 16)])
def test_dn_group_matches_oracle(P, N, c, G):
    rng = np.random.default_rng(P + 7 * N + G)
    f = np.float32
    theta0 = (rng.standard_normal(P) * 0.02).astype(f)
    dn = DelayedNesterov(theta0, 0.7, 0.9, N, c)
    # put the server in a mid-run state: a few events already applied
    t0 = 2
    for _ in range(t0):
        dn.event((rng.standard_normal(P) * 1e-3).astype(f))
    starts = [(rng.standard_normal(P) * 0.02).astype(f) for _ in range(G)]
    works = [s + (rng.standard_normal(P) * 1e-3).astype(f) for s in starts]
    th, m, de = _dev(dn.theta), _dev(dn.m), _dev(dn.delta)
    ts = [_dev(s) for s in starts]
    tw = [_dev(w) for w in works]
    lp = [torch.zeros(max(P, 1), dtype=torch.bfloat16, device=DEV) for _ in range(G)]
    A.k_dn_group(th, m, de, ts, tw, lp, N, t0, 0.7, 0.9, c, restart=True)
    torch.cuda.synchronize()
    for s, w in zip(starts, works):
        dn.event(s - w)
    tol = 2e-6
    if P:
        assert _rel(th.cpu().numpy(), dn.theta) < tol
        np.testing.assert_allclose(m.cpu().numpy(), dn.m, rtol=1e-5, atol=1e-9)
        np.testing.assert_allclose(de.cpu().numpy(), dn.delta, rtol=1e-5, atol=1e-9)
        for j in range(G):      # restart wrote the new theta everywhere
            assert torch.equal(ts[j], th) and torch.equal(tw[j], th)
            assert torch.equal(lp[j][:P], th.to(torch.bfloat16))


def test_dn_group_equals_single_events():
    P, N = 4096 * 3 + 8, 4
    rng = np.random.default_rng(0)
    f = np.float32
    base = [(rng.standard_normal(P) * 0.02).astype(f) for _ in range(3)]
    starts = [(rng.standard_normal(P) * 0.02).astype(f) for _ in range(5)]
    works = [s + (rng.standard_normal(P) * 1e-3).astype(f) for s in starts]
    a = [_dev(x) for x in base]
    b = [_dev(x) for x in base]
    A.k_dn_group(a[0], a[1], a[2], [_dev(s) for s in starts], [_dev(w) for w in works], None, N, 1, 0.7, 0.9)
    for j in range(5):
        A.k_dn_group(b[0], b[1], b[2], [_dev(starts[j])], [_dev(works[j])], None, N, 1 + j, 0.7, 0.9)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("P,Pd", [(0, 0), (3, 2), (1024, 1024), (4 * 256 * 19 + 2, 4 * 256 * 19 - 4), (1 << 20, (1 << 20) - 64)])
def test_adamw_matches_oracle(P, Pd):
    rng = np.random.default_rng(P)
    f = np.float32
    theta = (rng.standard_normal(P) * 0.02).astype(f)
    opt = AdamW(P, f, wd=0.1, n_decayed=Pd)
    th, m, v = _dev(theta), torch.zeros(max(P, 1), device=DEV)[:P], torch.zeros(max(P, 1), device=DEV)[:P]
    lp = torch.zeros(max(P, 1), dtype=torch.bfloat16, device=DEV)
    ref = theta.copy()
    for step in range(1, 6):
        g = (rng.standard_normal(P) * 10 ** rng.uniform(-6, 0)).astype(f)
        if P > 10:
            g[::7] = 0.0
        A.k_adamw(th, _dev(g), m, v, lp, Pd, step, 1e-3)
        opt.step(ref, g, 1e-3)
    torch.cuda.synchronize()
    if P:
        np.testing.assert_allclose(th.cpu().numpy(), ref, rtol=2e-6, atol=1e-9)
        np.testing.assert_allclose(m.cpu().numpy(), opt.m, rtol=1e-5, atol=1e-8)
        np.testing.assert_allclose(v.cpu().numpy(), opt.v, rtol=1e-5, atol=1e-15)
        assert torch.equal(lp[:P], th.to(torch.bfloat16))


@pytest.mark.parametrize("M,N,K", [(64, 64, 16), (70, 33, 19), (256, 192, 128), (1, 5, 300)])
@pytest.mark.parametrize("al,bl", [(0, 0), (0, 1), (1, 0), (1, 1)])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_gemm_generic(M, N, K, al, bl, dt):
    rng = np.random.default_rng(M * N + K)
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = rng.standard_normal((K, N)).astype(np.float32)
    ad = _dev(a if al == 0 else a.T.copy(), dt)
    bd = _dev(b if bl == 0 else b.T.copy(), dt)
    c = torch.empty(M, N, dtype=torch.float32, device=DEV)
    A.k_gemm(ad, bd, c, M, N, K, al, bl)
    torch.cuda.synchronize()
    ar = (ad.float().cpu().numpy() if al == 0 else ad.float().cpu().numpy().T).astype(np.float64)
    br = (bd.float().cpu().numpy() if bl == 0 else bd.float().cpu().numpy().T).astype(np.float64)
    np.testing.assert_allclose(c.cpu().numpy(), ar @ br, rtol=1e-5, atol=1e-4)


def _attention_case(B, S, h, dh, dt, use_mfma, scale=1.0):
    rng = np.random.default_rng(S + dh)
    d = h * dh
    qkv = _dev(rng.standard_normal((B * S, 3 * d)).astype(np.float32) * scale, dt)
    d_o = _dev(rng.standard_normal((B * S, d)).astype(np.float32) * 0.1, dt)
    o = torch.empty(B * S, d, dtype=dt, device=DEV)
    lse = torch.empty(B * h * S, dtype=torch.float32, device=DEV)
    dq = torch.empty_like(qkv)
    scratch = torch.empty(B * h * S, dtype=torch.float32, device=DEV)
    A.k_attention_fwd(qkv, o, lse, B, S, h, dh, use_mfma)
    A.k_attention_bwd(qkv, o, d_o, lse, scratch, dq, B, S, h, dh, use_mfma)
    torch.cuda.synchronize()
    x = qkv.float().cpu().numpy().astype(np.float64)
    split = lambda z: z.reshape(B, S, h, dh).transpose(0, 2, 1, 3)
    q, k, v = split(x[:, :d]), split(x[:, d:2 * d]), split(x[:, 2 * d:])
    oo, p = lm.attention_fwd(q, k, v)
    do4 = split(d_o.float().cpu().numpy().astype(np.float64))
    rdq, rdk, rdv = lm.attention_bwd(do4, q, k, v, p)
    merge = lambda z: z.transpose(0, 2, 1, 3).reshape(B * S, d)
    ref_dqkv = np.concatenate([merge(rdq), merge(rdk), merge(rdv)], axis=1)
    s = np.matmul(q, np.swapaxes(k, -1, -2)) / np.sqrt(dh)
    s = np.where(np.triu(np.ones((S, S), bool), 1), -np.inf, s)
    ref_lse = np.log(np.sum(np.exp(s - s.max(-1, keepdims=True)), -1)) + s.max(-1)
    return (o.float().cpu().numpy(), merge(oo), lse.cpu().numpy().reshape(B, h, S), ref_lse,
            dq.float().cpu().numpy(), ref_dqkv)


@pytest.mark.parametrize("B,S,h,dh", [(2, 32, 2, 32), (1, 70, 3, 64), (2, 130, 1, 64), (1, 1, 1, 32)])
@pytest.mark.parametrize("dt", [torch.float32, torch.bfloat16])
def test_attention_generic(B, S, h, dh, dt):
    o, ro, lse, rlse, dq, rdq = _attention_case(B, S, h, dh, dt, False)
    tol = 2e-5 if dt == torch.float32 else 2e-2
    assert _rel(o, ro) < tol
    np.testing.assert_allclose(lse, rlse, rtol=1e-5, atol=1e-5)
    assert _rel(dq, rdq) < tol


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (256, 256, 128), (512, 384, 192), (2048, 4096, 256), (4096, 512, 512)])
@pytest.mark.parametrize("al,bl", [(0, 0), (0, 1)])
@pytest.mark.parametrize("odt", [torch.float32, torch.bfloat16])
def test_gemm_mfma_forward_and_input_gradient_layouts(M, N, K, al, bl, odt):
    rng = np.random.default_rng(M + N + K)
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = rng.standard_normal((K, N)).astype(np.float32)
    ad = _dev(a, torch.bfloat16)
    bd = _dev(b if bl == 0 else b.T.copy(), torch.bfloat16)
    c = torch.full((M, N), float("nan"), dtype=odt, device=DEV)
    A.k_gemm(ad, bd, c, M, N, K, al, bl, use_mfma=True)
    torch.cuda.synchronize()
    ar = ad.float().cpu().numpy().astype(np.float64)
    br = bd.float().cpu().numpy().astype(np.float64)
    ref = ar @ (br if bl == 0 else br.T)
    got = c.float().cpu().numpy()
    if odt == torch.float32:
        np.testing.assert_allclose(got, ref, rtol=1e-4, atol=1e-3)
    else:
        np.testing.assert_allclose(got, ref, rtol=1e-2, atol=1e-2)


@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (256, 384, 4096), (512, 1536, 16384), (896, 3584, 2048)])
def test_gemm_mfma_weight_gradient_layout(M, N, K):
    rng = np.random.default_rng(M + N + K)
    x = rng.standard_normal((K, M)).astype(np.float32)        # stored [K, M]
    dy = rng.standard_normal((K, N)).astype(np.float32)       # stored [K, N]
    xd, dyd = _dev(x, torch.bfloat16), _dev(dy, torch.bfloat16)
    ref = xd.float().cpu().numpy().astype(np.float64).T @ dyd.float().cpu().numpy().astype(np.float64)
    ws = torch.empty(8 * M * N, dtype=torch.float32, device=DEV)      # room for 8 split-K partials
    for scratch in (None, ws):
        c = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        A.k_gemm(xd, dyd, c, M, N, K, 1, 0, use_mfma=True, ws=scratch)
        torch.cuda.synchronize()
        np.testing.assert_allclose(c.cpu().numpy(), ref, rtol=1e-4, atol=2e-3 * np.sqrt(K / 64))


def test_gemm_mfma_rejects_unsupported_shapes():
    a = torch.zeros(100, 64, dtype=torch.bfloat16, device=DEV)
    b = torch.zeros(64, 128, dtype=torch.bfloat16, device=DEV)
    c = torch.zeros(100, 128, dtype=torch.float32, device=DEV)
    with pytest.raises(A.AlsError):
        A.k_gemm(a, b, c, 100, 128, 64, 0, 0, use_mfma=True)
    with pytest.raises(A.AlsError):
        A.k_gemm(a.float(), b.float(), c, 128, 128, 64, 0, 0, use_mfma=True)


@pytest.mark.parametrize("B,S,h", [(2, 128, 2), (1, 256, 3), (1, 384, 1), (2, 512, 2), (1, 1024, 1)])
def test_attention_mfma(B, S, h):
    o, ro, lse, rlse, dq, rdq = _attention_case(B, S, h, 64, torch.bfloat16, True)
    assert _rel(o, ro) < 1e-2
    np.testing.assert_allclose(lse, rlse, rtol=1e-4, atol=1e-4)
    d = h * 64
    for nm, sl in (("dq", slice(0, d)), ("dk", slice(d, 2 * d)), ("dv", slice(2 * d, 3 * d))):
        assert _rel(dq[:, sl], rdq[:, sl]) < 1.5e-2, nm


@pytest.mark.parametrize("scale", [3.0, 0.05])
def test_attention_mfma_score_ranges(scale):
    """Scores with a standard deviation of 9 (the running reference point of the online softmax must
    move several times along a row, by more than its 2^8 slack) and nearly constant scores."""
    o, ro, lse, rlse, dq, rdq = _attention_case(2, 512, 2, 64, torch.bfloat16, True, scale=scale)
    assert np.isfinite(o).all() and np.isfinite(dq).all()
    assert _rel(o, ro) < 1e-2
    np.testing.assert_allclose(lse, rlse, rtol=1e-4, atol=1e-4)
    assert _rel(dq, rdq) < 2e-2


def test_attention_mfma_matches_generic_kernel_closely():
    # same bf16 inputs through both GPU kernels: they differ only by rounding of P to bf16
    B, S, h = 1, 256, 2
    o1, _, l1, _, g1, _ = _attention_case(B, S, h, 64, torch.bfloat16, True)
    o2, _, l2, _, g2, _ = _attention_case(B, S, h, 64, torch.bfloat16, False)
    assert _rel(o1, o2) < 1e-2 and _rel(g1, g2) < 1.5e-2
    np.testing.assert_allclose(l1, l2, rtol=1e-4, atol=1e-4)


@pytest.mark.timeout(900)
def test_outer_step_microbench_vector_full_size():
    """Benchmark configs[2]: 150M-element fp32 vector, 4 replicas, N = 4, one grouped pass ending
    on the momentum update, and one AdamW step, all compared element by element."""
    mb = I.OUTER_MICROBENCH
    P, G, N = mb["P"], 4, 4
    f = np.float32
    theta = I.normal_vector(P, [mb["seed"], 1], mb["sigma"])
    m = I.normal_vector(P, [mb["seed"], 2], 1e-3)
    delta = np.zeros(P, f)
    dn = DelayedNesterov(theta, mb["outer_lr"], mb["outer_beta"], N, 0.0)
    dn.m[...] = m
    th, md, dd = _dev(theta), _dev(m), _dev(delta)
    ts, tw = [], []
    for j in range(G):
        start = I.normal_vector(P, [mb["seed"], 10 + j], mb["sigma"])
        work = start + I.normal_vector(P, [mb["seed"], 30 + j], mb["drift_sigma"])
        ts.append(_dev(start))
        tw.append(_dev(work))
        dn.event(start - work)
        del start, work
    A.k_dn_group(th, md, dd, ts, tw, None, N, 0, mb["outer_lr"], mb["outer_beta"], 0.0, restart=True)
    torch.cuda.synchronize()
    assert dn.t == 4 and not dn.delta.any()
    assert _rel(th.cpu().numpy(), dn.theta) < 2e-6
    np.testing.assert_allclose(md.cpu().numpy(), dn.m, rtol=1e-5, atol=1e-9)
    assert not dd.any().item()
    assert torch.equal(tw[3], th) and torch.equal(ts[0], th)
    del ts, tw, dn
    # AdamW on the same vector
    g = I.normal_vector(P, [mb["seed"], 50], 1e-3)
    ref = theta.copy()
    opt = AdamW(P, f, wd=0.1, n_decayed=P - 4096)
    opt.m[...] = m
    opt.v[...] = m * m
    opt.n = 6
    am, av = _dev(m), _dev(m * m)
    th2 = _dev(theta)
    lp = torch.empty(P, dtype=torch.bfloat16, device=DEV)
    A.k_adamw(th2, _dev(g), am, av, lp, P - 4096, 7, 1e-3)
    opt.step(ref, g, 1e-3)
    torch.cuda.synchronize()
    np.testing.assert_allclose(th2.cpu().numpy(), ref, rtol=2e-6, atol=1e-9)
    np.testing.assert_allclose(av.cpu().numpy(), opt.v, rtol=1e-5, atol=1e-15)
    assert torch.equal(lp, th2.to(torch.bfloat16))


@pytest.mark.parametrize("mfma", [False, True])
def test_gemm_epilogues(mfma):
    M, N, K = 256, 384, 128
    rng = np.random.default_rng(0)
    a = _dev(rng.standard_normal((M, K)).astype(np.float32), torch.bfloat16)
    w = _dev(rng.standard_normal((K, N)).astype(np.float32) * 0.2, torch.bfloat16)
    acc = a.float().cpu().numpy().astype(np.float64) @ w.float().cpu().numpy().astype(np.float64)
    # residual
    r = _dev(rng.standard_normal((M, N)).astype(np.float32))
    c = torch.empty(M, N, dtype=torch.float32, device=DEV)
    A.k_gemm_ex(a, w, c, M, N, K, 0, 0, mfma, epi=1, R=r)
    torch.cuda.synchronize()
    np.testing.assert_allclose(c.cpu().numpy(), acc + r.cpu().numpy(), rtol=1e-4, atol=1e-3)
    # GELU pair: C = gelu'(acc), C2 = gelu(acc)
    gp = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    gv = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    A.k_gemm_ex(a, w, gp, M, N, K, 0, 0, mfma, epi=2, C2=gv)
    torch.cuda.synchronize()
    np.testing.assert_allclose(gv.float().cpu().numpy(), lm.gelu_fwd(acc), rtol=1e-2, atol=1e-2)
    np.testing.assert_allclose(gp.float().cpu().numpy(), lm.gelu_grad(acc), rtol=1e-2, atol=1e-2)
    # multiply by a saved derivative (input-gradient layout: B stored [N, K])
    u = _dev(rng.standard_normal((M, N)).astype(np.float32), torch.bfloat16)
    wt = w.t().contiguous()
    d = torch.empty(M, N, dtype=torch.bfloat16, device=DEV)
    A.k_gemm_ex(a, wt, d, M, N, K, 0, 1, mfma, epi=3, U=u)
    torch.cuda.synchronize()
    np.testing.assert_allclose(d.float().cpu().numpy(), acc * u.float().cpu().numpy(), rtol=1e-2, atol=2e-2)


@pytest.mark.parametrize("seed", range(40))
def test_gemm_mfma_random_shapes_layouts_and_tiles(seed):
    """Random tile-aligned shapes in every operand layout the step uses, under a randomly forced
    tile / buffering variant (or the automatic choice), with and without split-K scratch."""
    rng = np.random.default_rng([seed, 0x6E])
    al, bl = [(0, 0), (0, 1), (1, 0)][int(rng.integers(0, 3))]
    tile = [(0, 0, 0), (256, 256, 2), (256, 128, 2), (256, 128, 1), (128, 128, 2), (128, 128, 1), (128, 128, 3),
            (256, 256, 4), (256, 256, 5)][int(rng.integers(0, 9))]
    # (buffering codes 4, 5 = the 256 x 256 kernel with two wavefront groups in alternating phases, 5 with
    # operands loaded straight into LDS where the layout allows; both mask partial tiles)
    unit_m, unit_n = (128, 128) if tile[2] >= 4 else (max(tile[0], 128), max(tile[1], 128))
    M, N = unit_m * int(rng.integers(1, 5)), unit_n * int(rng.integers(1, 5))
    K = 64 * int(rng.integers(1, 48))
    out_bf16 = bool(rng.integers(0, 2)) and al == 0
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = rng.standard_normal((K, N)).astype(np.float32)
    ad = _dev(a if al == 0 else a.T.copy(), torch.bfloat16)
    bd = _dev(b if bl == 0 else b.T.copy(), torch.bfloat16)
    ar = ad.float().cpu().numpy().astype(np.float64)
    br = bd.float().cpu().numpy().astype(np.float64)
    ref = (ar if al == 0 else ar.T) @ (br if bl == 0 else br.T)
    ws = torch.empty(int(rng.integers(1, 9)) * M * N, dtype=torch.float32, device=DEV) if (al == 1 and rng.integers(0, 2)) else None
    c = torch.full((M, N), float("nan"), dtype=torch.bfloat16 if out_bf16 else torch.float32, device=DEV)
    try:
        A.lib.als_k_set_gemm_tile(*tile)
        A.k_gemm(ad, bd, c, M, N, K, al, bl, use_mfma=True, ws=ws)
        torch.cuda.synchronize()
    finally:
        A.lib.als_k_set_gemm_tile(0, 0, 0)
    what = f"M{M} N{N} K{K} layouts {al}{bl} tile {tile} bf16 out {out_bf16} scratch {None if ws is None else ws.numel() // (M * N)}"
    if out_bf16:
        np.testing.assert_allclose(c.float().cpu().numpy(), ref, rtol=1e-2, atol=1e-2 * np.sqrt(K / 64), err_msg=what)
    else:
        np.testing.assert_allclose(c.cpu().numpy(), ref, rtol=1e-4, atol=2e-3 * np.sqrt(K / 64), err_msg=what)


def test_gemm_mfma_tile_variants_agree():
    """Every tile / buffering variant of the MFMA GEMM gives the same product."""
    M, N, K = 512, 512, 256
    rng = np.random.default_rng(1)
    a = _dev(rng.standard_normal((M, K)).astype(np.float32), torch.bfloat16)
    b = _dev(rng.standard_normal((K, N)).astype(np.float32), torch.bfloat16)
    ref = a.float().cpu().numpy().astype(np.float64) @ b.float().cpu().numpy().astype(np.float64)
    try:
        for tile in [(256, 256, 2), (256, 128, 2), (256, 128, 1), (128, 128, 2), (128, 128, 1), (128, 128, 3), (256, 256, 4), (256, 256, 5)]:
            A.lib.als_k_set_gemm_tile(*tile)
            c = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
            A.k_gemm(a, b, c, M, N, K, 0, 0, use_mfma=True)
            torch.cuda.synchronize()
            np.testing.assert_allclose(c.cpu().numpy(), ref, rtol=1e-4, atol=2e-3, err_msg=str(tile))
    finally:
        A.lib.als_k_set_gemm_tile(0, 0, 0)


@pytest.mark.parametrize("tile", [(128, 128, 1), (128, 128, 2), (256, 256, 4), (256, 256, 5)])
def test_gemm_epilogues_under_every_mfma_kernel(tile):
    """Residual, GELU pair, multiply-by-saved-derivative and plain bf16 / fp32 stores under each MFMA
    kernel (4 = the 256 x 256 kernel with two wavefront groups in alternating phases, 5 = its
    direct-to-LDS form), on a shape whose last tiles are partial in both directions for the 256-wide
    kernels (384 x 640) and whose K (192) is three slices."""
    M, N, K = 384, 640, 192
    rng = np.random.default_rng(7)
    a = _dev(rng.standard_normal((M, K)).astype(np.float32), torch.bfloat16)
    w = _dev(rng.standard_normal((K, N)).astype(np.float32) * 0.2, torch.bfloat16)
    acc = a.float().cpu().numpy().astype(np.float64) @ w.float().cpu().numpy().astype(np.float64)
    r = _dev(rng.standard_normal((M, N)).astype(np.float32))
    u = _dev(rng.standard_normal((M, N)).astype(np.float32), torch.bfloat16)
    wt = w.t().contiguous()
    try:
        A.lib.als_k_set_gemm_tile(*tile)
        c = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        A.k_gemm_ex(a, w, c, M, N, K, 0, 0, True, epi=1, R=r)
        gp = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        gv = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        A.k_gemm_ex(a, w, gp, M, N, K, 0, 0, True, epi=2, C2=gv)
        d = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        A.k_gemm_ex(a, wt, d, M, N, K, 0, 1, True, epi=3, U=u)
        pb = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
        A.k_gemm(a, w, pb, M, N, K, 0, 0, use_mfma=True)
        pf = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        A.k_gemm(a, wt, pf, M, N, K, 0, 1, use_mfma=True)
        torch.cuda.synchronize()
    finally:
        A.lib.als_k_set_gemm_tile(0, 0, 0)
    np.testing.assert_allclose(c.cpu().numpy(), acc + r.cpu().numpy(), rtol=1e-4, atol=1e-3)
    np.testing.assert_allclose(gv.float().cpu().numpy(), lm.gelu_fwd(acc), rtol=1e-2, atol=1e-2)
    np.testing.assert_allclose(gp.float().cpu().numpy(), lm.gelu_grad(acc), rtol=1e-2, atol=1e-2)
    np.testing.assert_allclose(d.float().cpu().numpy(), acc * u.float().cpu().numpy(), rtol=1e-2, atol=2e-2)
    np.testing.assert_allclose(pb.float().cpu().numpy(), acc, rtol=1e-2, atol=1e-2)
    np.testing.assert_allclose(pf.cpu().numpy(), acc, rtol=1e-4, atol=1e-3)


@pytest.mark.parametrize("tile", [(256, 256, 4), (256, 256, 5)])
@pytest.mark.parametrize("M,N,K,scratch", [(256, 256, 64, 0), (384, 896, 4096, 8), (896, 2688, 16384, 6), (128, 512, 1024, 4)])
def test_pingpong_gemm_weight_gradient_shapes(tile, M, N, K, scratch):
    """The 256 x 256 kernels on the weight-gradient layout (both operands contraction-strided): a
    single K slice, partial tiles in both directions, split along K when scratch for the partials
    is given, and a product with fewer rows than a tile."""
    rng = np.random.default_rng(M + N + K)
    x = _dev(rng.standard_normal((K, M)).astype(np.float32), torch.bfloat16)
    dy = _dev(rng.standard_normal((K, N)).astype(np.float32), torch.bfloat16)
    ref = x.float().cpu().numpy().astype(np.float64).T @ dy.float().cpu().numpy().astype(np.float64)
    ws = torch.empty(scratch * M * N, dtype=torch.float32, device=DEV) if scratch else None
    c = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    try:
        A.lib.als_k_set_gemm_tile(*tile)
        A.k_gemm(x, dy, c, M, N, K, 1, 0, use_mfma=True, ws=ws)
        torch.cuda.synchronize()
    finally:
        A.lib.als_k_set_gemm_tile(0, 0, 0)
    np.testing.assert_allclose(c.cpu().numpy(), ref, rtol=1e-4, atol=2e-3 * np.sqrt(K / 64))


@pytest.mark.parametrize("tile", [(256, 256, 4), (256, 256, 5)])
@pytest.mark.parametrize("layout", [(0, 0), (0, 1), (1, 0)])
@pytest.mark.parametrize("M,N", [(384, 512), (128, 256), (512, 384), (384, 384), (896, 896)])
def test_pingpong_gemm_half_tiles(tile, layout, M, N):
    """Half tiles of the 256 x 256 kernels: a dead lower row half (the wavefront groups then own the
    row halves), a dead right column half, and the corner tile with both, in every operand layout;
    dead wavefronts multiply nothing and every live element is exact to fp32 accumulation."""
    al, bl = layout
    K = 320
    rng = np.random.default_rng([M, N, al, bl])
    a = rng.standard_normal((M, K)).astype(np.float32)
    b = rng.standard_normal((K, N)).astype(np.float32)
    ad = _dev(a if al == 0 else a.T.copy(), torch.bfloat16)
    bd = _dev(b if bl == 0 else b.T.copy(), torch.bfloat16)
    ar = ad.float().cpu().numpy().astype(np.float64)
    br = bd.float().cpu().numpy().astype(np.float64)
    ref = (ar if al == 0 else ar.T) @ (br if bl == 0 else br.T)
    c = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
    try:
        A.lib.als_k_set_gemm_tile(*tile)
        A.k_gemm(ad, bd, c, M, N, K, al, bl, use_mfma=True)
        torch.cuda.synchronize()
    finally:
        A.lib.als_k_set_gemm_tile(0, 0, 0)
    np.testing.assert_allclose(c.cpu().numpy(), ref, rtol=1e-4, atol=4e-3)


@pytest.mark.parametrize("M,N,K,al,bl", [(896, 2688, 8192, 1, 0), (1024, 896, 1792, 0, 1), (768, 640, 896, 0, 0)])
def test_pingpong_forms_agree_bit_for_bit(M, N, K, al, bl):
    """The register-staged and the direct-to-LDS form of the 256 x 256 kernel multiply the same
    fragments in the same order (and split K into the same ranges, added in the same order), so
    their fp32 results are equal bit for bit, masked half tiles included."""
    rng = np.random.default_rng([M, N, K])
    a = _dev(rng.standard_normal((K, M) if al else (M, K)).astype(np.float32), torch.bfloat16)
    b = _dev(rng.standard_normal((N, K) if bl else (K, N)).astype(np.float32), torch.bfloat16)
    ws = torch.empty(8 * M * N, dtype=torch.float32, device=DEV) if al else None
    out = []
    for code in (4, 5):
        c = torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV)
        try:
            A.lib.als_k_set_gemm_tile(256, 256, code)
            A.k_gemm(a, b, c, M, N, K, al, bl, use_mfma=True, ws=ws)
            torch.cuda.synchronize()
        finally:
            A.lib.als_k_set_gemm_tile(0, 0, 0)
        out.append(c)
    assert torch.isfinite(out[0]).all()
    assert torch.equal(out[0], out[1])


def _grouped_case(shapes, K, seed):
    rng = np.random.default_rng(seed)
    Xs = [_dev(rng.standard_normal((K, M)).astype(np.float32), torch.bfloat16) for M, _ in shapes]
    dYs = [_dev(rng.standard_normal((K, N)).astype(np.float32), torch.bfloat16) for _, N in shapes]
    Cs = [torch.full((M, N), float("nan"), dtype=torch.float32, device=DEV) for M, N in shapes]
    ws = torch.empty(A.k_gemm_dw_grouped_ws_bytes([m for m, _ in shapes], [n for _, n in shapes]), dtype=torch.uint8, device=DEV)
    A.k_gemm_dw_grouped(Xs, dYs, Cs, K, ws)
    torch.cuda.synchronize()
    for X, dY, Cm in zip(Xs, dYs, Cs):
        ref = X.float().cpu().numpy().astype(np.float64).T @ dY.float().cpu().numpy().astype(np.float64)
        np.testing.assert_allclose(Cm.cpu().numpy(), ref, rtol=1e-4, atol=2e-3 * np.sqrt(K / 64))
    return Xs, dYs, Cs, ws


@pytest.mark.parametrize("shapes,K", [
    ([(256, 256)], 64),                                              # one tile, one slice: no split possible
    ([(128, 384), (384, 128), (256, 640)], 1024),                    # 7 tiles, all in the split remainder, half tiles
    ([(896, 896), (896, 2688), (3584, 896), (896, 3584)] * 2, 512),  # 344 tiles: one whole round and a split remainder
    ([(512, 2048), (2048, 512), (512, 512), (512, 1536)] * 6, 2048), # 288 tiles, the 20M-class layer set
    ([(1024, 1024)] * 16, 256),                                      # exactly one round of whole tiles, nothing split
    ([(768, 768)] * 50, 128),                                        # 450 tiles, 2 slices each: one round, then 194 unsplit tiles
    ([(896, 3584), (3584, 896)] * 6, 256),                           # 672 tiles: two rounds and 160 unsplit tiles, half tiles
])
def test_grouped_weight_gradients(shapes, K):
    """Every product of the grouped launch against a float64 product of the same bf16 operands:
    whole tiles, K-split remainder tiles with their reduction, half tiles, and the boundaries of the
    plan (a single tile, an exact round)."""
    _grouped_case(shapes, K, seed=[len(shapes), K])


def test_grouped_weight_gradients_are_reproducible():
    """Two launches on the same operands give the same bits (partial tiles are added in slot order)."""
    shapes = [(896, 2688), (896, 896), (896, 3584), (3584, 896)] * 3
    Xs, dYs, Cs, ws = _grouped_case(shapes, 1024, seed=7)
    first = [c.clone() for c in Cs]
    for c in Cs:
        c.fill_(float("nan"))
    A.k_gemm_dw_grouped(Xs, dYs, Cs, 1024, ws)
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(first, Cs))
