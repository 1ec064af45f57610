"""Pins for the oracle's language model: loss value and hand-derived gradient (CPU only)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import als_inputs as I
from oracle import lm

CFG = dict(L=2, d=16, h=2, ff=40, V=23, S=6, norm_eps=1e-5)
# attention width h * dh = 24 on a hidden size of 16 (the paper's larger models have 16 heads of
# 64 on 896)
CFG_WIDE = dict(L=2, d=16, h=3, dh=8, ff=40, V=23, S=6, norm_eps=1e-5)
# layer normalisation (gain only) instead of RMS normalisation
CFG_LN = dict(CFG, norm="layer")
BOTH = pytest.mark.parametrize("CFG", [CFG, CFG_WIDE, CFG_LN], ids=["square", "wide", "layernorm"])


def _theta(cfg, seed=0, sigma=0.3, dtype=np.float64):
    th = I.theta0(lm.param_layout(cfg), seed, sigma).astype(dtype)
    # move the gains off 1 so their gradient paths are exercised
    rng = np.random.default_rng(seed + 1)
    nd = lm.n_decayed(cfg)
    th[nd:] += 0.2 * rng.standard_normal(th.size - nd)
    return th


def _tokens(cfg, B=3, seed=0):
    return I.zipf_tokens(np.random.default_rng(seed), cfg["V"], (B, cfg["S"] + 1))


def test_layout_counts():
    cfg = I.workload("tiny")
    L, d, ff, V, S = cfg["L"], cfg["d"], cfg["ff"], cfg["V"], cfg["S"]
    assert lm.n_params(cfg) == 2 * V * d + S * d + L * (4 * d * d + 2 * d * ff) + (2 * L + 1) * d
    assert lm.n_params(cfg) - lm.n_decayed(cfg) == (2 * L + 1) * d
    assert lm.n_params(I.workload("lm20m")) == 27_531_776


def test_layout_counts_wide_attention():
    c = CFG_WIDE
    shapes = {n: sh for n, sh, _ in lm.param_layout(c)}
    assert shapes["Wqkv0"] == (16, 72) and shapes["Wo1"] == (24, 16)
    assert lm.n_params(c) == lm.n_params(CFG) + c["L"] * (16 * 3 * 8 + 8 * 16)
    # the paper's 150M row: 12 layers, 896 hidden, 16 heads of 64
    p = dict(L=12, d=896, h=16, dh=64, ff=3584, V=32000, S=256)
    assert lm.n_params(p) == 2 * 32000 * 896 + 256 * 896 + 12 * (896 * 3072 + 1024 * 896 + 2 * 896 * 3584) + 25 * 896


@BOTH
def test_gradient_matches_central_finite_differences_every_tensor(CFG):
    th = _theta(CFG)
    tok = _tokens(CFG)
    _, grad = lm.loss_and_grad(th, tok, CFG)
    rng = np.random.default_rng(0)
    off = 0
    h = 1e-5
    for name, shape, _ in lm.param_layout(CFG):
        n = int(np.prod(shape))
        for j in rng.choice(n, size=min(n, 6), replace=False):
            e = np.zeros_like(th)
            e[off + j] = h
            fd = (lm.forward(th + e, tok, CFG, keep=False)[0] - lm.forward(th - e, tok, CFG, keep=False)[0]) / (2 * h)
            assert grad[off + j] == pytest.approx(fd, rel=2e-6, abs=1e-9), (name, j)
        off += n
    # embedding rows of tokens that never occur as inputs get exactly zero gradient
    g = lm.views(grad, CFG)
    unused = sorted(set(range(CFG["V"])) - set(tok[:, :-1].reshape(-1).tolist()))
    assert unused and not g["E"][unused].any()


@BOTH
def test_directional_derivative_full_vector(CFG):
    th = _theta(CFG, seed=4)
    tok = _tokens(CFG, seed=4)
    _, grad = lm.loss_and_grad(th, tok, CFG)
    v = np.random.default_rng(9).standard_normal(th.size)
    h = 1e-6
    fd = (lm.forward(th + h * v, tok, CFG, keep=False)[0] - lm.forward(th - h * v, tok, CFG, keep=False)[0]) / (2 * h)
    assert float(grad @ v) == pytest.approx(fd, rel=1e-6)


def _torch_loss(theta_t, tok, cfg):
    """The same model written independently with library ops and autograd."""
    L, d, h, ff, V, S = (cfg[k] for k in ("L", "d", "h", "ff", "V", "S"))
    dh = cfg.get("dh", d // h)
    off = 0

    def take(*shape):
        nonlocal off
        n = int(np.prod(shape))
        t = theta_t[off:off + n].view(*shape)
        off += n
        return t

    E, Ppos = take(V, d), take(S, d)
    mats = [(take(d, 3 * h * dh), take(h * dh, d), take(d, ff), take(ff, d)) for _ in range(L)]
    Wout = take(d, V)
    gains = [(take(d), take(d)) for _ in range(L)]
    gf = take(d)
    tok = torch.as_tensor(tok, dtype=torch.long)
    B = tok.shape[0]
    x = F.embedding(tok[:, :S], E) + Ppos
    if cfg.get("norm", "rms") == "layer":
        norm = lambda t, g: F.layer_norm(t, (d,), g, None, cfg["norm_eps"])
    else:
        norm = lambda t, g: F.rms_norm(t, (d,), g, cfg["norm_eps"])
    for (Wqkv, Wo, W1, W2), (g1, g2) in zip(mats, gains):
        a = norm(x, g1)
        q, k, v = (a @ Wqkv).split(h * dh, dim=-1)
        q, k, v = (z.view(B, S, h, dh).transpose(1, 2) for z in (q, k, v))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
        x = x + o.transpose(1, 2).reshape(B, S, h * dh) @ Wo
        b = norm(x, g2)
        x = x + F.gelu(b @ W1, approximate="tanh") @ W2
    logits = norm(x, gf) @ Wout
    return F.cross_entropy(logits.view(B * S, V), tok[:, 1:].reshape(-1))


@BOTH
def test_loss_and_gradient_match_library_autograd(CFG):
    th = _theta(CFG, seed=2)
    tok = _tokens(CFG, B=4, seed=2)
    loss, grad = lm.loss_and_grad(th, tok, CFG)
    tt = torch.tensor(th, requires_grad=True)
    tl = _torch_loss(tt, tok, CFG)
    tl.backward()
    assert float(loss) == pytest.approx(float(tl.detach()), rel=1e-12)
    np.testing.assert_allclose(grad, tt.grad.numpy(), rtol=1e-9, atol=1e-13)


def test_float32_path_close_to_float64():
    cfg = I.workload("tiny")
    th = I.theta0(lm.param_layout(cfg), 0)
    tok = _tokens(cfg, B=cfg["B"])
    l32, g32 = lm.loss_and_grad(th, tok, cfg)
    l64, g64 = lm.loss_and_grad(th.astype(np.float64), tok, cfg)
    assert g32.dtype == np.float32
    assert float(l32) == pytest.approx(float(l64), rel=1e-6)
    assert np.linalg.norm(g32 - g64) / np.linalg.norm(g64) < 1e-5


@pytest.mark.parametrize("name", ["tiny", "mini_f32"])
def test_initial_loss_is_log_vocab(name):
    cfg = I.workload(name)
    th = I.theta0(lm.param_layout(cfg), 0)
    tok = I.TokenStream(0, 0, cfg["B"], cfg["S"], cfg["V"]).take(1)[0]
    loss, _ = lm.forward(th, tok, cfg, keep=False)
    assert float(loss) == pytest.approx(math.log(cfg["V"]), abs=0.05)
    # with a zero output matrix the loss is exactly log V
    v = lm.views(th, cfg)
    v["Wout"][...] = 0
    assert float(lm.forward(th, tok, cfg, keep=False)[0]) == pytest.approx(math.log(cfg["V"]), rel=1e-6)


def test_causality():
    th = _theta(CFG, seed=5)
    tok = _tokens(CFG, B=2, seed=5)
    _, c0 = lm.forward(th, tok, CFG)
    tok2 = tok.copy()
    j = 4
    tok2[:, j] = (tok2[:, j] + 1) % CFG["V"]
    _, c1 = lm.forward(th, tok2, CFG)
    S = CFG["S"]
    a = c0["logits"].reshape(2, S, -1)
    b = c1["logits"].reshape(2, S, -1)
    np.testing.assert_array_equal(a[:, :j], b[:, :j])
    assert np.abs(a[:, j:] - b[:, j:]).max() > 1e-6


def test_pieces_against_library():
    rng = np.random.default_rng(0)
    u = rng.standard_normal(50) * 3
    np.testing.assert_allclose(lm.gelu_fwd(u), F.gelu(torch.tensor(u), approximate="tanh").numpy(), atol=1e-14)
    ut = torch.tensor(u, requires_grad=True)
    F.gelu(ut, approximate="tanh").sum().backward()
    np.testing.assert_allclose(lm.gelu_grad(u), ut.grad.numpy(), atol=1e-13)
    x = rng.standard_normal((5, 8))
    g = rng.standard_normal(8)
    y, _ = lm.rmsnorm_fwd(x, g, 1e-5)
    np.testing.assert_allclose(y, F.rms_norm(torch.tensor(x), (8,), torch.tensor(g), 1e-5).numpy(), atol=1e-14)
    # layer normalisation (gain, no bias): forward against the library, backward against its
    # autograd, and two closed forms of its input gradient: it sums to zero over a row, and along
    # the centred row it is eps rstd^2 <dy g, xhat> (zero but for eps: y ignores the row's scale)
    x = rng.standard_normal((5, 8)) + 0.7
    y, rstd = lm.layernorm_fwd(x, g, 1e-5)
    xt = torch.tensor(x, requires_grad=True)
    gt = torch.tensor(g, requires_grad=True)
    yt = F.layer_norm(xt, (8,), gt, None, 1e-5)
    np.testing.assert_allclose(y, yt.detach().numpy(), atol=1e-14)
    dy = rng.standard_normal((5, 8))
    yt.backward(torch.tensor(dy))
    dx, dg = lm.layernorm_bwd(dy, x, rstd, g)
    np.testing.assert_allclose(dx, xt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dg, gt.grad.numpy(), atol=1e-13)
    np.testing.assert_allclose(dx.sum(axis=1), 0.0, atol=1e-13)
    xc = x - x.mean(axis=1, keepdims=True)
    np.testing.assert_allclose((dx * xc).sum(axis=1), 1e-5 * rstd[:, 0] ** 2 * (dy * g * xc * rstd).sum(axis=1), atol=1e-14)


def test_bf16_operand_rounding_matches_the_library_conversion_and_perturbs_little():
    """oracle.lm.round_bf16 equals the library's float32 -> bfloat16 -> float32 conversion (round to
    nearest, ties to even) on random values, exact ties, subnormal-sized and large values; the
    oracle with bf16-rounded operands stays within a few 1e-3 of the plain one (8 mantissa bits),
    and is not identical to it."""
    import torch
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(100000).astype(np.float32) * np.float32(3.0),
                        np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-30, -7.5e-20]),
                        # exact ties: 1 + (2k+1) 2^-8 lies midway between two bfloat16 values
                        (1.0 + (2 * np.arange(64) + 1) * 2.0 ** -8).astype(np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(lm.round_bf16(x).view(np.uint32), want.view(np.uint32))
    w = dict(I.workload("tiny"))
    theta = I.theta0(lm.param_layout(w), 0)
    tok = I.TokenStream(0, 0, w["B"], w["S"], w["V"]).take(1)[0]
    l0, g0 = lm.loss_and_grad(theta.copy(), tok, w)
    l1, g1 = lm.loss_and_grad(theta.copy(), tok, dict(w, operand_rounding="bf16"))
    assert l0 != l1 and abs(l0 - l1) / abs(l0) < 2e-3
    rel = np.linalg.norm(g1.astype(np.float64) - g0) / np.linalg.norm(g0.astype(np.float64))
    assert 1e-4 < rel < 2e-2
