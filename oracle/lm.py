"""Decoder-only transformer language model: next-token cross-entropy loss and its gradient.

The paper fixes only "decoder-only transformer" (appendix, Network Architecture / model
configuration table) and "cross entropy loss for next token prediction" (Background, Eq. 1).
The reading used here: pre-norm blocks with RMSNorm (eps 1e-5, learned gain), causal
multi-head softmax attention with scale 1/sqrt(dh), tanh-GELU feed-forward, learned
absolute position embeddings, no biases, no dropout, untied input/output embeddings, loss
averaged over all B*S predicted positions.

Flat parameter vector layout (all row-major):
  E [V,d], Ppos [S,d], then per layer Wqkv [d,3a] (columns q|k|v, head-major inside each;
  a = attention width = h * head width, equal to d unless cfg["dh"] is set), Wo [a,d],
  W1 [d,ff], W2 [ff,d]; then Wout [d,V]; then all gains: per layer g1 [d], g2 [d];
  finally gf [d].  Everything before the gains is weight-decayed, the gains are not.
"""
from __future__ import annotations

import math
import numpy as np


def attention_width(cfg):
    """h * head width; the head width is cfg["dh"] if given (the paper's 60M and 150M models
    use 16 heads of 64 on a hidden size of 896), else d / h."""
    return cfg["h"] * (cfg.get("dh") or cfg["d"] // cfg["h"])


def param_layout(cfg):
    """List of (name, shape, kind); kind is "matrix" (decayed) or "gain" (not decayed)."""
    L, d, ff, V, S = cfg["L"], cfg["d"], cfg["ff"], cfg["V"], cfg["S"]
    da = attention_width(cfg)
    out = [("E", (V, d), "matrix"), ("Ppos", (S, d), "matrix")]
    for l in range(L):
        out += [(f"Wqkv{l}", (d, 3 * da), "matrix"), (f"Wo{l}", (da, d), "matrix"),
                (f"W1{l}", (d, ff), "matrix"), (f"W2{l}", (ff, d), "matrix")]
    out.append(("Wout", (d, V), "matrix"))
    for l in range(L):
        out += [(f"g1{l}", (d,), "gain"), (f"g2{l}", (d,), "gain")]
    out.append(("gf", (d,), "gain"))
    return out


def n_params(cfg):
    return sum(int(np.prod(s)) for _, s, _ in param_layout(cfg))


def n_decayed(cfg):
    return sum(int(np.prod(s)) for _, s, k in param_layout(cfg) if k == "matrix")


def views(flat, cfg):
    """Dict name -> reshaped view into the flat vector."""
    out, off = {}, 0
    for name, shape, _ in param_layout(cfg):
        n = int(np.prod(shape))
        out[name] = flat[off:off + n].reshape(shape)
        off += n
    assert off == flat.size
    return out


# ---------------------------------------------------------------------------------------
# pieces
# ---------------------------------------------------------------------------------------
def rmsnorm_fwd(x, g, eps):
    rstd = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + x.dtype.type(eps))
    return x * rstd * g, rstd


def rmsnorm_bwd(dy, x, rstd, g):
    xhat = x * rstd
    dg = np.sum((dy * xhat).reshape(-1, x.shape[-1]), axis=0)
    dxhat = dy * g
    dx = rstd * (dxhat - xhat * np.mean(dxhat * xhat, axis=-1, keepdims=True))
    return dx, dg


def layernorm_fwd(x, g, eps):
    """Layer normalisation with a gain and no bias (the model has no biases anywhere):
    y = (x - mean) / sqrt(var + eps) * g, var = mean((x - mean)^2)."""
    xc = x - np.mean(x, axis=-1, keepdims=True)
    rstd = 1.0 / np.sqrt(np.mean(xc * xc, axis=-1, keepdims=True) + x.dtype.type(eps))
    return xc * rstd * g, rstd


def layernorm_bwd(dy, x, rstd, g):
    xhat = (x - np.mean(x, axis=-1, keepdims=True)) * rstd
    dg = np.sum((dy * xhat).reshape(-1, x.shape[-1]), axis=0)
    dxhat = dy * g
    dx = rstd * (dxhat - np.mean(dxhat, axis=-1, keepdims=True)
                 - xhat * np.mean(dxhat * xhat, axis=-1, keepdims=True))
    return dx, dg


def _norm(cfg):
    """(forward, backward) of the configured normalisation: cfg["norm"] = "rms" (default) or
    "layer"."""
    kind = cfg.get("norm", "rms")
    if kind == "rms":
        return rmsnorm_fwd, rmsnorm_bwd
    if kind == "layer":
        return layernorm_fwd, layernorm_bwd
    raise ValueError(f"unknown norm {kind!r}")


_GELU_A = math.sqrt(2.0 / math.pi)
_GELU_B = 0.044715


def gelu_fwd(u):
    t = u.dtype.type
    return t(0.5) * u * (t(1.0) + np.tanh(t(_GELU_A) * (u + t(_GELU_B) * u * u * u)))


def gelu_grad(u):
    t = u.dtype.type
    th = np.tanh(t(_GELU_A) * (u + t(_GELU_B) * u * u * u))
    inner = t(_GELU_A) * (t(1.0) + t(3.0 * _GELU_B) * u * u)
    return t(0.5) * (t(1.0) + th) + t(0.5) * u * (t(1.0) - th * th) * inner


def round_bf16(x):
    """float32 array rounded to the nearest bfloat16 value (ties to even), returned as float32:
    add 0x7FFF plus the lowest kept mantissa bit to the bit pattern and clear the low 16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + (((u >> 16) & np.uint32(1)) + np.uint32(0x7FFF))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def _operands(cfg):
    """What happens to the two operands of every matrix product before it is formed.  By default
    nothing.  cfg["operand_rounding"] = "bf16" rounds both to bfloat16 (the product itself is still
    accumulated in the array dtype, float32): the precision policy "bf16 in, fp32 accumulate"
    applied to the oracle's own products, used to measure how far a correct implementation with
    bf16 operands may sit from the plain float32 result."""
    kind = cfg.get("operand_rounding")
    if kind is None:
        return lambda x: x
    if kind == "bf16":
        return round_bf16
    raise ValueError(f"unknown operand rounding {kind!r}")


def attention_fwd(q, k, v, rnd=lambda x: x):
    """q,k,v [B,h,S,dh] -> o [B,h,S,dh], p [B,h,S,S] (causal softmax probabilities)."""
    S, dh = q.shape[2], q.shape[3]
    s = np.matmul(rnd(q), np.swapaxes(rnd(k), -1, -2)) * q.dtype.type(1.0 / math.sqrt(dh))
    mask = np.triu(np.ones((S, S), dtype=bool), k=1)
    s = np.where(mask, -np.inf, s)
    s = s - np.max(s, axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / np.sum(p, axis=-1, keepdims=True)
    return np.matmul(rnd(p), rnd(v)), p


def attention_bwd(do, q, k, v, p, rnd=lambda x: x):
    dh = q.shape[3]
    dv = np.matmul(np.swapaxes(rnd(p), -1, -2), rnd(do))
    dp = np.matmul(rnd(do), np.swapaxes(rnd(v), -1, -2))
    ds = p * (dp - np.sum(dp * p, axis=-1, keepdims=True))
    ds = ds * q.dtype.type(1.0 / math.sqrt(dh))
    dq = np.matmul(rnd(ds), rnd(k))
    dk = np.matmul(np.swapaxes(rnd(ds), -1, -2), rnd(q))
    return dq, dk, dv


def _split_heads(x, B, S, h):
    return x.reshape(B, S, h, -1).transpose(0, 2, 1, 3)


def _merge_heads(x):
    B, h, S, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * S, h * dh)


# ---------------------------------------------------------------------------------------
# loss and gradient
# ---------------------------------------------------------------------------------------
def forward(theta, tokens, cfg, keep=True):
    """tokens int [B,S+1].  Returns (loss, cache).  Also cache["logits"] [B*S,V]."""
    p = views(theta, cfg)
    L, d, h, S = cfg["L"], cfg["d"], cfg["h"], cfg["S"]
    da = attention_width(cfg)
    eps = cfg["norm_eps"]
    norm_fwd, _ = _norm(cfg)
    rnd = _operands(cfg)
    B = tokens.shape[0]
    assert tokens.shape[1] == S + 1
    inp, tgt = tokens[:, :S], tokens[:, 1:].reshape(-1)
    x = (p["E"][inp] + p["Ppos"][None, :, :]).reshape(B * S, d)
    layers = []
    for l in range(L):
        a, rstd1 = norm_fwd(x, p[f"g1{l}"], eps)
        qkv = rnd(a) @ rnd(p[f"Wqkv{l}"])
        q = _split_heads(qkv[:, :da], B, S, h)
        k = _split_heads(qkv[:, da:2 * da], B, S, h)
        v = _split_heads(qkv[:, 2 * da:], B, S, h)
        o4, prob = attention_fwd(q, k, v, rnd)
        o = _merge_heads(o4)
        xm = x + rnd(o) @ rnd(p[f"Wo{l}"])
        b, rstd2 = norm_fwd(xm, p[f"g2{l}"], eps)
        u = rnd(b) @ rnd(p[f"W1{l}"])
        gl = gelu_fwd(u)
        xn = xm + rnd(gl) @ rnd(p[f"W2{l}"])
        if keep:
            layers.append(dict(x=x, a=a, rstd1=rstd1, q=q, k=k, v=v, prob=prob, o=o, xm=xm,
                               b=b, rstd2=rstd2, u=u, gl=gl))
        x = xn
    xf, rstdf = norm_fwd(x, p["gf"], eps)
    logits = rnd(xf) @ rnd(p["Wout"])
    mx = np.max(logits, axis=-1, keepdims=True)
    lse = mx[:, 0] + np.log(np.sum(np.exp(logits - mx), axis=-1))
    T = B * S
    loss = np.mean(lse - logits[np.arange(T), tgt])
    cache = dict(inp=inp, tgt=tgt, layers=layers, x=x, xf=xf, rstdf=rstdf, logits=logits,
                 lse=lse, B=B)
    return loss, cache


def backward(theta, cache, cfg):
    """Flat gradient of the mean loss, same layout as theta."""
    p = views(theta, cfg)
    grad = np.zeros_like(theta)
    g = views(grad, cfg)
    L, d, h, S = cfg["L"], cfg["d"], cfg["h"], cfg["S"]
    B = cache["B"]
    T = B * S
    rnd = _operands(cfg)
    logits, lse, tgt = cache["logits"], cache["lse"], cache["tgt"]
    dlogits = np.exp(logits - lse[:, None])
    dlogits[np.arange(T), tgt] -= 1.0
    dlogits = dlogits * theta.dtype.type(1.0 / T)
    g["Wout"][...] = rnd(cache["xf"]).T @ rnd(dlogits)
    dxf = rnd(dlogits) @ rnd(p["Wout"]).T
    _, norm_bwd = _norm(cfg)
    dx, dgf = norm_bwd(dxf, cache["x"], cache["rstdf"], p["gf"])
    g["gf"][...] = dgf
    for l in reversed(range(L)):
        c = cache["layers"][l]
        g[f"W2{l}"][...] = rnd(c["gl"]).T @ rnd(dx)
        dgl = rnd(dx) @ rnd(p[f"W2{l}"]).T
        du = dgl * gelu_grad(c["u"])
        g[f"W1{l}"][...] = rnd(c["b"]).T @ rnd(du)
        db = rnd(du) @ rnd(p[f"W1{l}"]).T
        dxm_n, dg2 = norm_bwd(db, c["xm"], c["rstd2"], p[f"g2{l}"])
        g[f"g2{l}"][...] = dg2
        dxm = dx + dxm_n
        g[f"Wo{l}"][...] = rnd(c["o"]).T @ rnd(dxm)
        do = _split_heads(rnd(dxm) @ rnd(p[f"Wo{l}"]).T, B, S, h)
        dq, dk, dv = attention_bwd(do, c["q"], c["k"], c["v"], c["prob"], rnd)
        dqkv = np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=1)
        g[f"Wqkv{l}"][...] = rnd(c["a"]).T @ rnd(dqkv)
        da = rnd(dqkv) @ rnd(p[f"Wqkv{l}"]).T
        dx_n, dg1 = norm_bwd(da, c["x"], c["rstd1"], p[f"g1{l}"])
        g[f"g1{l}"][...] = dg1
        dx = dxm + dx_n
    dx3 = dx.reshape(B, S, d)
    g["Ppos"][...] = dx3.sum(axis=0)
    np.add.at(g["E"], cache["inp"].reshape(-1), dx)
    return grad


def loss_and_grad(theta, tokens, cfg):
    loss, cache = forward(theta, tokens, cfg)
    return loss, backward(theta, cache, cfg)
