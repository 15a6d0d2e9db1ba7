"""CPU oracle of the second layer family (the LLaMA models of the paper's Table III): one tensor-model-parallel
rank's share of a pre-RMSNorm layer with rotary position embedding and a SwiGLU feed-forward block.

TEST INFRASTRUCTURE ONLY, like layer_oracle.py (whose attention and dropout-mask definitions it calls); nothing on
the product path may import it.  The method is the same as for the GPT layer -- Megatron's partition with the
paper's two forward and two backward reduction points per layer (Sec. II, Sec. IV-B Eq. (1)) -- so the oracle is
again the plain definition of the layer written for one rank in the general form "attention inner width hp, FFN
inner width fp, the other ranks' partial sums handed in as peers".

The paper names the model family and no formula.  Readings (each pinned in tests/test_oracle_llama.py):
  RMSNorm          y = g * x / sqrt(mean(x^2) + eps), no mean subtraction, no bias (Zhang & Sennrich 2019)
  rotary embedding pairs (i, i + d/2) of a head rotate by pos * theta^(-2i/d), theta = 10000, pos = index of the token
                   in its sequence ("rotate-half" pairing); applied to Q and K
  SwiGLU           f = silu(v2 Wg) * (v2 Wu), silu(z) = z * sigmoid(z); column-parallel Wg, Wu, row-parallel W2
  no biases; the two hidden dropouts of the GPT layer stay available (LLaMA itself trains with p = 0)
Backward is the chain rule by hand for the loss <dy, y>.
"""
from __future__ import annotations

import torch

from .layer_oracle import _Rounder, attention_bwd, attention_dropout_factor, attention_fwd, dropout_keep_mask

LLAMA_BF16_OPERAND_SITES = ("u", "qkv", "P", "A", "v2", "gu", "f", "dZ2", "dGU", "dZ1", "dA", "dS", "dqkv")


def rms_norm_fwd(x, gamma, eps):
    rstd = 1.0 / torch.sqrt((x * x).mean(dim=1, keepdim=True) + eps)
    return gamma * (x * rstd), rstd


def rms_norm_bwd(dy, x, rstd, gamma):
    xhat = x * rstd
    g = dy * gamma
    dx = rstd * (g - xhat * (g * xhat).mean(dim=1, keepdim=True))
    return dx, (dy * xhat).sum(dim=0)


def rope_angles(seq: int, d: int, theta: float, dtype):
    """[seq, d/2] rotation angles pos * theta^(-2i/d)."""
    i = torch.arange(d // 2, dtype=torch.float64)
    inv = theta ** (-2.0 * i / d)
    return (torch.arange(seq, dtype=torch.float64)[:, None] * inv[None, :]).to(dtype)


def rope_apply(t, batch: int, seq: int, d: int, theta: float, inverse: bool = False):
    """t: [batch*seq, nh*d], rows batch-major.  Element pair (i, i + d/2) of every head is rotated by the token's angle;
    inverse=True rotates back (the transpose of the rotation: what the gradient needs)."""
    M, w = t.shape
    nh = w // d
    ang = rope_angles(seq, d, theta, t.dtype)
    cos, sin = torch.cos(ang), torch.sin(ang)
    if inverse:
        sin = -sin
    x = t.reshape(batch, seq, nh, d)
    x1, x2 = x[..., : d // 2], x[..., d // 2:]
    c, s = cos[None, :, None, :], sin[None, :, None, :]
    return torch.cat([x1 * c - x2 * s, x2 * c + x1 * s], dim=-1).reshape(M, w)


def silu(z):
    return z * torch.sigmoid(z)


def silu_grad(z):
    sg = torch.sigmoid(z)
    return sg * (1.0 + z * (1.0 - sg))


def rank_layer_forward(p: dict, x, *, batch: int, seq: int, head_dim: int, causal: bool = True, dropout_p: float = 0.0,
                       seed: int = 0, layer: int = 0, eps: float = 1e-5, theta: float = 10000.0, peers: dict | None = None,
                       bf16_sites=(), attn_dropout_p: float = 0.0, head0: int = 0, n_heads_total: int | None = None):
    """`p`: wq, wk, wv [h,hp], wo [hp,h], wg, wu [h,fp], w2 [fp,h], ln1_g, ln2_g [h].  Returns (y, saved)."""
    rb = _Rounder(bf16_sites)
    peers = peers or {}
    M, h = x.shape
    assert M == batch * seq
    hp = p["wq"].shape[1]
    nh = hp // head_dim
    dt = x.dtype
    c = 1.0 / (1.0 - dropout_p)
    D1 = torch.from_numpy(dropout_keep_mask(seed, layer, 0, M, h, dropout_p)).to(dt)
    D2 = torch.from_numpy(dropout_keep_mask(seed, layer, 1, M, h, dropout_p)).to(dt)

    u, rstd1 = rms_norm_fwd(x, p["ln1_g"], eps)
    u = rb("u", u)
    q = rb("qkv", rope_apply(rb("qkv", u @ p["wq"]), batch, seq, head_dim, theta))
    k = rb("qkv", rope_apply(rb("qkv", u @ p["wk"]), batch, seq, head_dim, theta))
    v = rb("qkv", u @ p["wv"])
    drop = attention_dropout_factor(seed, layer, batch, seq, n_heads_total or nh, head0, nh, attn_dropout_p)
    A, P = attention_fwd(q, k, v, batch, seq, nh, head_dim, causal, rb, drop)
    Z1r = A @ p["wo"]
    Z1 = Z1r + peers["fwd_attn"] if peers.get("fwd_attn") is not None else Z1r
    x1 = x + D1 * Z1 * c
    v2, rstd2 = rms_norm_fwd(x1, p["ln2_g"], eps)
    v2 = rb("v2", v2)
    gate, up = v2 @ p["wg"], v2 @ p["wu"]
    f = rb("f", silu(gate) * up)
    gate, up = rb("gu", gate), rb("gu", up)
    Z2r = f @ p["w2"]
    Z2 = Z2r + peers["fwd_ffn"] if peers.get("fwd_ffn") is not None else Z2r
    y = x1 + D2 * Z2 * c
    saved = dict(x=x, u=u, rstd1=rstd1, q=q, k=k, v=v, P=P, A=A, Z1r=Z1r, Z1=Z1, x1=x1, rstd2=rstd2, v2=v2, gate=gate, up=up,
                 f=f, Z2r=Z2r, Z2=Z2, y=y, D1=D1, D2=D2, c=c, batch=batch, seq=seq, head_dim=head_dim, theta=theta, drop=drop)
    return y, saved


def rank_layer_backward(p: dict, saved: dict, dy, *, peers: dict | None = None, bf16_sites=()):
    """Returns (dx, grads, inter); `peers` may hold 'bwd_ffn' / 'bwd_attn' (Eq. (1): the gradient passes through a
    forward reduction unchanged, the column-parallel inputs' gradients are summed over ranks)."""
    rb = _Rounder(bf16_sites)
    peers = peers or {}
    s = saved
    b, seq, d, c, theta = s["batch"], s["seq"], s["head_dim"], s["c"], s["theta"]
    nh = p["wq"].shape[1] // d
    g = {}
    dZ2 = rb("dZ2", s["D2"] * dy * c)
    dx1 = dy.clone()
    dF = dZ2 @ p["w2"].t()
    g["w2"] = s["f"].t() @ dZ2
    dgate = rb("dGU", dF * s["up"] * silu_grad(s["gate"]))
    dup = rb("dGU", dF * silu(s["gate"]))
    g["wg"] = s["v2"].t() @ dgate
    g["wu"] = s["v2"].t() @ dup
    dV2r = dgate @ p["wg"].t() + dup @ p["wu"].t()
    dV2 = dV2r + peers["bwd_ffn"] if peers.get("bwd_ffn") is not None else dV2r
    dn2, g["ln2_g"] = rms_norm_bwd(dV2, s["x1"], s["rstd2"], p["ln2_g"])
    dx1 = dx1 + dn2
    dZ1 = rb("dZ1", s["D1"] * dx1 * c)
    dA = rb("dA", dZ1 @ p["wo"].t())
    g["wo"] = s["A"].t() @ dZ1
    dq, dk, dv = attention_bwd(dA, s["q"], s["k"], s["v"], s["P"], b, seq, nh, d, rb, s.get("drop"))
    dq = rb("dqkv", rope_apply(dq, b, seq, d, theta, inverse=True))     # back through the rotation
    dk = rb("dqkv", rope_apply(dk, b, seq, d, theta, inverse=True))
    for n, dd in (("q", dq), ("k", dk), ("v", dv)):
        g["w" + n] = s["u"].t() @ dd
    dUr = dq @ p["wq"].t() + dk @ p["wk"].t() + dv @ p["wv"].t()
    dU = dUr + peers["bwd_attn"] if peers.get("bwd_attn") is not None else dUr
    dn1, g["ln1_g"] = rms_norm_bwd(dU, s["x"], s["rstd1"], p["ln1_g"])
    dx = dx1 + dn1
    inter = dict(dZ2=dZ2, dgate=dgate, dup=dup, dV2r=dV2r, dV2=dV2, dx1=dx1, dZ1=dZ1, dA=dA, dq=dq, dk=dk, dv=dv, dUr=dUr, dU=dU)
    return dx, g, inter


def model_forward_backward(layers: list, x, dy, cfg: dict, *, seed: int = 0, dtype=torch.float64, bf16_sites=(),
                           want_backward: bool = True, head0: int = 0):
    """Stack of layers, as layer_oracle.model_forward_backward."""
    import numpy as np
    d = cfg["hidden"] // cfg["n_heads"]
    tp = [{k: torch.from_numpy(np.ascontiguousarray(v)).to(dtype) for k, v in l.items()} for l in layers]
    cur = torch.from_numpy(np.ascontiguousarray(x)).to(dtype)
    saved = []
    for li, p in enumerate(tp):
        cur, sv = rank_layer_forward(p, cur, batch=cfg["batch"], seq=cfg["seq"], head_dim=d, causal=bool(cfg["causal"]),
                                     dropout_p=cfg["dropout_p"], seed=seed, layer=li, theta=cfg.get("rope_theta", 10000.0),
                                     bf16_sites=bf16_sites, attn_dropout_p=cfg.get("attn_dropout_p", 0.0), head0=head0,
                                     n_heads_total=cfg["n_heads"])
        saved.append(sv)
    out = dict(y=cur, saved=saved)
    if want_backward:
        g = torch.from_numpy(np.ascontiguousarray(dy)).to(dtype)
        grads, inters = [None] * len(tp), [None] * len(tp)
        for li in reversed(range(len(tp))):
            g, grads[li], inters[li] = rank_layer_backward(tp[li], saved[li], g, bf16_sites=bf16_sites)
        out.update(dx=g, grads=grads, inter=inters)
    return out
