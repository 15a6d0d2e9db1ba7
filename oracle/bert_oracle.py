"""CPU oracle of the third layer family (the BERT models of the paper's Table III): one tensor-model-parallel rank's
share of a post-LayerNorm layer, non-causal by default.

TEST INFRASTRUCTURE ONLY, like layer_oracle.py (whose operator definitions it calls); nothing on the product path
may import it.  Same method as for the other families -- Megatron's partition, two forward and two backward
reduction points per layer (Sec. II; Sec. IV-B Eq. (1)) -- so the oracle is the plain definition of the layer for
one rank in the general form "attention inner width hp, FFN inner width fp, peers' partial sums handed in".

Reading (the paper names the model family only): the original Transformer / BERT block,
    s1 = x  + dropout(attention(x) Wo + bo),   x1 = LayerNorm1(s1)
    s2 = x1 + dropout(gelu(x1 W1 + b1) W2 + b2),   y = LayerNorm2(s2)
with the LayerNorm, GeLU, dropout-mask and softmax readings of the GPT layer.  The linear maps read the bf16 copy of
their fp32 input (x, x1).  Backward is the chain rule by hand for the loss <dy, y>.
"""
from __future__ import annotations

import numpy as np
import torch

from .layer_oracle import (_Rounder, attention_bwd, attention_dropout_factor, attention_fwd, dropout_keep_mask, gelu_fwd, gelu_grad,
                           layer_norm_bwd, layer_norm_fwd)

BERT_BF16_OPERAND_SITES = ("u", "qkv", "P", "A", "v2", "pre", "f", "dZ2", "dG", "dZ1", "dA", "dS", "dqkv")


def rank_layer_forward(p: dict, x, *, batch: int, seq: int, head_dim: int, causal: bool = False, dropout_p: float = 0.0,
                       seed: int = 0, layer: int = 0, eps: float = 1e-5, peers: dict | None = None, bf16_sites=(), attn_dropout_p: float = 0.0, head0: int = 0,
                       n_heads_total: int | None = None):
    """`p` as in layer_oracle.rank_layer_forward; ln1_* normalise the attention block's output, ln2_* the FFN block's."""
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

    u = rb("u", x)
    q = rb("qkv", u @ p["wq"] + p["bq"])
    k = rb("qkv", u @ p["wk"] + p["bk"])
    v = rb("qkv", u @ p["wv"] + p["bv"])
    drop = attention_dropout_factor(seed, layer, batch, seq, n_heads_total or nh, head0, nh, attn_dropout_p)
    A, P = attention_fwd(q, k, v, batch, seq, nh, head_dim, causal, rb, drop)
    Z1r = A @ p["wo"]
    Z1 = Z1r + peers["fwd_attn"] if peers.get("fwd_attn") is not None else Z1r
    s1 = x + D1 * (Z1 + p["bo"]) * c
    x1, mu1, rstd1 = layer_norm_fwd(s1, p["ln1_g"], p["ln1_b"], eps)
    v2 = rb("v2", x1)
    pre = v2 @ p["w1"] + p["b1"]
    f = rb("f", gelu_fwd(pre, True))
    pre = rb("pre", pre)
    Z2r = f @ p["w2"]
    Z2 = Z2r + peers["fwd_ffn"] if peers.get("fwd_ffn") is not None else Z2r
    s2 = x1 + D2 * (Z2 + p["b2"]) * c
    y, mu2, rstd2 = layer_norm_fwd(s2, p["ln2_g"], p["ln2_b"], eps)
    saved = dict(x=x, u=u, q=q, k=k, v=v, P=P, A=A, Z1r=Z1r, Z1=Z1, s1=s1, mu1=mu1, rstd1=rstd1, x1=x1, v2=v2, pre=pre, f=f, Z2r=Z2r,
                 Z2=Z2, s2=s2, mu2=mu2, rstd2=rstd2, y=y, D1=D1, D2=D2, c=c, batch=batch, seq=seq, head_dim=head_dim, drop=drop)
    return y, saved


def rank_layer_backward(p: dict, saved: dict, dy, *, peers: dict | None = None, bf16_sites=()):
    """Returns (dx, grads, inter); `peers` may hold 'bwd_ffn' / 'bwd_attn'."""
    rb = _Rounder(bf16_sites)
    peers = peers or {}
    s = saved
    b, seq, d, c = s["batch"], s["seq"], s["head_dim"], s["c"]
    nh = p["wq"].shape[1] // d
    g = {}
    ds2, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dy, s["s2"], s["mu2"], s["rstd2"], p["ln2_g"])
    dZ2 = rb("dZ2", s["D2"] * ds2 * c)
    g["b2"] = dZ2.sum(dim=0)
    dF = dZ2 @ p["w2"].t()
    g["w2"] = s["f"].t() @ dZ2
    dG = rb("dG", dF * gelu_grad(s["pre"], True))
    g["b1"] = dG.sum(dim=0)
    dV2r = dG @ p["w1"].t()
    g["w1"] = s["v2"].t() @ dG
    dV2 = dV2r + peers["bwd_ffn"] if peers.get("bwd_ffn") is not None else dV2r
    dx1 = ds2 + dV2                                           # residual branch + FFN input
    ds1, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(dx1, s["s1"], s["mu1"], s["rstd1"], p["ln1_g"])
    dZ1 = rb("dZ1", s["D1"] * ds1 * c)
    g["bo"] = dZ1.sum(dim=0)
    dA = rb("dA", dZ1 @ p["wo"].t())
    g["wo"] = s["A"].t() @ dZ1
    dq, dk, dv = attention_bwd(dA, s["q"], s["k"], s["v"], s["P"], b, seq, nh, d, rb, s.get("drop"))
    for n, dd in (("q", dq), ("k", dk), ("v", dv)):
        g["w" + n] = s["u"].t() @ dd
        g["b" + n] = dd.sum(dim=0)
    dUr = dq @ p["wq"].t() + dk @ p["wk"].t() + dv @ p["wv"].t()
    dU = dUr + peers["bwd_attn"] if peers.get("bwd_attn") is not None else dUr
    dx = ds1 + dU
    inter = dict(ds2=ds2, dZ2=dZ2, dG=dG, dV2r=dV2r, dV2=dV2, dx1=dx1, ds1=ds1, dZ1=dZ1, dA=dA, dq=dq, dk=dk, dv=dv, dUr=dUr, dU=dU)
    return dx, g, inter


def model_forward_backward(layers: list, x, dy, cfg: dict, *, seed: int = 0, dtype=torch.float64, bf16_sites=(),
                           want_backward: bool = True, head0: int = 0):
    d = cfg["hidden"] // cfg["n_heads"]
    tp = [{k: torch.from_numpy(np.ascontiguousarray(v)).to(dtype) for k, v in l.items()} for l in layers]
    cur = torch.from_numpy(np.ascontiguousarray(x)).to(dtype)
    saved = []
    for li, p in enumerate(tp):
        cur, sv = rank_layer_forward(p, cur, batch=cfg["batch"], seq=cfg["seq"], head_dim=d, causal=bool(cfg["causal"]),
                                     dropout_p=cfg["dropout_p"], seed=seed, layer=li, bf16_sites=bf16_sites,
                                     attn_dropout_p=cfg.get("attn_dropout_p", 0.0), head0=head0, n_heads_total=cfg["n_heads"])
        saved.append(sv)
    out = dict(y=cur, saved=saved)
    if want_backward:
        g = torch.from_numpy(np.ascontiguousarray(dy)).to(dtype)
        grads, inters = [None] * len(tp), [None] * len(tp)
        for li in reversed(range(len(tp))):
            g, grads[li], inters[li] = rank_layer_backward(tp[li], saved[li], g, bf16_sites=bf16_sites)
        out.update(dx=g, grads=grads, inter=inters)
    return out
