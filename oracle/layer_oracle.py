"""CPU oracle: one tensor-model-parallel rank's share of a pre-LN GPT transformer layer.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module; only
tests, the smoke check and the bench's cpu_baseline leg do.  It shares no code with
the HIP path.

What it computes.  The method (Oases' schedule over Megatron's partition) reaches
exactly the result of the unsharded layer: the schedule only reorders independent
sub-batch operators (Sec. IV-A: the order may change, the results may not) and the partition only
splits weight matrices by column or by row, with an AllReduce y = sum_i x_i whose
input gradient equals its output gradient (Sec. IV-B, Eq. (1)).  So the oracle is the
plain definition of the layer, written for *one rank* in the general form

    attention inner width hp = (local heads) * d,  FFN inner width fp,

with the sum of the other ranks' partial results handed in as `peers`.  The unsharded
layer is the special case hp = h, fp = 4h, peers = None; a rank of a t-way partition
is the case hp = h/t, fp = 4h/t with sliced weights (Sec. II, "Tensor model
parallelism": column split -> AllReduce in backward, row split -> AllReduce in
forward).  There is no blocking, fusion, sub-batching or reordering here: every step
is one plain tensor expression; `torch.matmul` on CPU is the only library primitive.
Backward is the chain rule written out by hand (no autograd).

Optional dropout on the attention probabilities (`attn_dropout_p`, off in the benchmark
configurations): a byte-granular Philox mask on (sequence, global head, query, key), see
attention_dropout_factor.

Readings where the paper is silent (it names no per-operator formula): pre-LN layer,
LayerNorm with biased variance and eps = 1e-5, tanh-form GeLU, biases on all four
linear maps with the row-parallel biases added once after the reduction, two hidden
dropouts (after projection+bias and after FC2+bias) whose keep mask is a function of
the *unsharded* element index through Philox4x32-10 (Salmon et al., SC'11), softmax
scale 1/sqrt(d), causal mask j <= i, loss phi = <dy, y>.

Parity pins (tests/test_oracle_*.py): Philox known-answer vectors, fp64 central finite
differences, torch autograd over library layer_norm / scaled_dot_product_attention /
gelu as an independent derivation, closed forms (causal row 0, zero weights, s = 1),
Megatron shard-sum identities.  The `bf16_sites` option (rounding of named tensors) is
an estimate of the storage-format error floor, not part of the definition; it is pinned
by tests/test_oracle_floor.py (rounding on the bit pattern, where each site rounds, what
its consumers read).
"""
from __future__ import annotations

import math

import numpy as np
import torch

# ----------------------------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3", SC'11)
# ----------------------------------------------------------------------------------------------
_PHILOX_M0 = np.uint64(0xD2511F53)
_PHILOX_M1 = np.uint64(0xCD9E8D57)
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds of Philox-4x32 on arrays of counters (uint32 values held in uint64 arrays).
    Returns the four 32-bit output words."""
    c0 = np.asarray(c0, dtype=np.uint64)
    c1 = np.asarray(c1, dtype=np.uint64)
    c2 = np.asarray(c2, dtype=np.uint64)
    c3 = np.asarray(c3, dtype=np.uint64)
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for rnd in range(10):
        p0 = _PHILOX_M0 * c0          # 64-bit product of two 32-bit values
        p1 = _PHILOX_M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        n0 = hi1 ^ c1 ^ np.uint64(k0)
        n2 = hi0 ^ c3 ^ np.uint64(k1)
        c0, c1, c2, c3 = n0, lo1, n2, lo0
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return c0, c1, c2, c3


def dropout_threshold(p: float) -> int:
    """Integer drop threshold on the top 24 bits of a Philox word: keep iff (word >> 8) >= T."""
    return int(round(p * (1 << 24)))


def dropout_keep_mask(seed: int, layer: int, site: int, n_rows: int, h: int, p: float,
                      row0: int = 0) -> np.ndarray:
    """Keep mask [n_rows, h] (bool) of dropout `site` (0 = after the attention block, 1 = after the
    FFN) in `layer`, for global token rows row0 .. row0+n_rows-1 of the unsharded [M, h] activation.

    Element e = row*h + col draws word (e mod 4) of Philox4x32-10 with key (seed lo32, seed hi32)
    and counter (q lo32, q hi32, site, layer), q = e div 4.  The element index is global, so the
    mask does not depend on the TP degree, the rank or the sub-batch split."""
    if p <= 0.0:
        return np.ones((n_rows, h), dtype=bool)
    assert h % 4 == 0
    e0 = row0 * h
    q = (np.arange(n_rows * h // 4, dtype=np.uint64) + np.uint64(e0 // 4))
    w = philox4x32_10(q & _MASK32, q >> np.uint64(32), np.full_like(q, site), np.full_like(q, layer),
                      seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack(w, axis=1).reshape(n_rows, h)           # word j of counter q -> element 4q + j
    return (words >> np.uint64(8)) >= np.uint64(dropout_threshold(p))


# ----------------------------------------------------------------------------------------------
# Operators
# ----------------------------------------------------------------------------------------------
def layer_norm_fwd(x, gamma, beta, eps):
    mu = x.mean(dim=1, keepdim=True)
    var = ((x - mu) ** 2).mean(dim=1, keepdim=True)          # biased variance
    rstd = 1.0 / torch.sqrt(var + eps)
    return gamma * ((x - mu) * rstd) + beta, mu, rstd


def layer_norm_bwd(dy, x, mu, rstd, gamma):
    xhat = (x - mu) * rstd
    g = dy * gamma
    dx = rstd * (g - g.mean(dim=1, keepdim=True) - xhat * (g * xhat).mean(dim=1, keepdim=True))
    return dx, (dy * xhat).sum(dim=0), dy.sum(dim=0)


_GELU_C0 = math.sqrt(2.0 / math.pi)
_GELU_C1 = 0.044715


def gelu_fwd(x, tanh_form=True):
    if tanh_form:
        return 0.5 * x * (1.0 + torch.tanh(_GELU_C0 * (x + _GELU_C1 * x ** 3)))
    return 0.5 * x * (1.0 + torch.erf(x / math.sqrt(2.0)))


def gelu_grad(x, tanh_form=True):
    if tanh_form:
        t = torch.tanh(_GELU_C0 * (x + _GELU_C1 * x ** 3))
        return 0.5 * (1.0 + t) + 0.5 * x * (1.0 - t * t) * _GELU_C0 * (1.0 + 3.0 * _GELU_C1 * x * x)
    return 0.5 * (1.0 + torch.erf(x / math.sqrt(2.0))) + x * torch.exp(-0.5 * x * x) / math.sqrt(2.0 * math.pi)


def _bf16(t):
    return t.to(torch.bfloat16).to(t.dtype)


class _Rounder:
    def __init__(self, sites):
        self.sites = frozenset(sites or ())

    def __call__(self, name, t):
        return _bf16(t) if name in self.sites else t


# every tensor a bf16-MFMA implementation must hold in bf16 (format-floor estimate)
BF16_OPERAND_SITES = ("u", "qkv", "P", "A", "v2", "pre", "f", "dZ2", "dG", "dZ1", "dA", "dS", "dqkv")


def attention_dropout_threshold(p: float) -> int:
    """Drop threshold on one byte of a Philox word: keep iff byte >= T.  The rate is thereby quantised to T/256."""
    return int(round(p * 256))


def attention_dropout_factor(seed: int, layer: int, batch: int, seq: int, n_heads_total: int, head0: int, nh_local: int,
                             p: float):
    """Dropout on the attention probabilities: the factor keep / (1 - T/256), as a [batch, nh_local, seq, seq] fp64
    tensor (query index third, key index last), or None if the quantised rate is 0.

    The mask is a function of (sequence b, global head, query position q, key position k): the 4 x 4 block
    (q div 4, k div 4) draws one Philox4x32-10 output with key (seed lo32, seed hi32) and counter
    (k div 4, q div 4, b * n_heads_total + head, layer | 2^31); element (q, k) takes byte (k mod 4) of word (q mod 4),
    low byte first.  Global head index: the mask does not depend on the TP degree, the rank or the sub-batch split."""
    T = attention_dropout_threshold(p)
    if T <= 0:
        return None
    nb = (seq + 3) // 4
    b_i, h_i, q4, k4 = np.meshgrid(np.arange(batch, dtype=np.uint64), np.arange(nh_local, dtype=np.uint64) + np.uint64(head0),
                                   np.arange(nb, dtype=np.uint64), np.arange(nb, dtype=np.uint64), indexing="ij")
    w = philox4x32_10(k4.ravel(), q4.ravel(), (b_i * np.uint64(n_heads_total) + h_i).ravel(),
                      np.full(k4.size, (layer & 0x7FFFFFFF) | 0x80000000, dtype=np.uint64), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack(w, axis=1).reshape(batch, nh_local, nb, nb, 4)                       # [.., q4, k4, q mod 4]
    bytes_ = np.stack([(words >> np.uint64(8 * j)) & np.uint64(0xFF) for j in range(4)], axis=-1)   # [.., q4, k4, q mod 4, k mod 4]
    keep = (bytes_ >= np.uint64(T)).transpose(0, 1, 2, 4, 3, 5).reshape(batch, nh_local, 4 * nb, 4 * nb)[:, :, :seq, :seq]
    return torch.from_numpy(keep.astype(np.float64) * (256.0 / (256.0 - T)))


def _heads(t, b, s, nh, d):
    """[b*s, nh*d] -> [b, nh, s, d]"""
    return t.reshape(b, s, nh, d).permute(0, 2, 1, 3)


def _unheads(t, b, s, nh, d):
    return t.permute(0, 2, 1, 3).reshape(b * s, nh * d)


def attention_fwd(q, k, v, batch, seq, nh, d, causal, rb=None, drop=None):
    """Softmax attention per (batch item, head) on [batch*seq, nh*d] matrices.  Returns (A, P).  `drop`: optional
    [batch, nh, seq, seq] dropout factor on the probabilities (P itself is returned undropped)."""
    rb = rb or _Rounder(())
    qh, kh, vh = (_heads(t, batch, seq, nh, d) for t in (q, k, v))
    S = (qh @ kh.transpose(2, 3)) / math.sqrt(d)                      # [b, nh, s, s]
    if causal:
        i = torch.arange(seq)
        S = S.masked_fill(i[None, :] > i[:, None], float("-inf"))     # key j visible iff j <= i
    S = S - S.max(dim=3, keepdim=True).values
    P = torch.exp(S)
    P = P / P.sum(dim=3, keepdim=True)
    Pd = P if drop is None else P * drop.to(P.dtype)
    A = rb("A", _unheads(rb("P", Pd) @ vh, batch, seq, nh, d))        # [M, nh*d]
    return A, P


def attention_bwd(dA, q, k, v, P, batch, seq, nh, d, rb=None, drop=None):
    """Gradients of attention_fwd's inputs for the output gradient dA (softmax' written out)."""
    rb = rb or _Rounder(())
    qh, kh, vh, dAh = (_heads(t, batch, seq, nh, d) for t in (q, k, v, dA))
    dP = dAh @ vh.transpose(2, 3)
    Pd = P
    if drop is not None:               # A = (P * drop) V: the factor multiplies both the path to V and the path to P
        dP = dP * drop.to(P.dtype)
        Pd = P * drop.to(P.dtype)
    dvh = rb("P", Pd).transpose(2, 3) @ dAh
    dS = rb("dS", P * (dP - (dP * P).sum(dim=3, keepdim=True)))
    dqh = (dS @ kh) / math.sqrt(d)
    dkh = (dS.transpose(2, 3) @ qh) / math.sqrt(d)
    return tuple(rb("dqkv", _unheads(t, batch, seq, nh, d)) for t in (dqh, dkh, dvh))


def rank_layer_forward(p: dict, x, *, batch: int, seq: int, head_dim: int, causal: bool,
                       dropout_p: float = 0.0, seed: int = 0, layer: int = 0, eps: float = 1e-5,
                       gelu_tanh: bool = True, peers: dict | None = None, bf16_sites=(), attn_dropout_p: float = 0.0,
                       head0: int = 0, n_heads_total: int | None = None):
    """Forward of one rank's share.  `p` holds torch tensors wq,wk,wv [h,hp], bq,bk,bv [hp], wo [hp,h],
    bo [h], w1 [h,fp], b1 [fp], w2 [fp,h], b2 [h], ln1_g, ln1_b, ln2_g, ln2_b [h]; x is [batch*seq, h].
    `peers` may hold 'fwd_attn' / 'fwd_ffn': the sum of the other ranks' partial results at the two
    forward reduction points.  Returns (y, saved)."""
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

    u, mu1, rstd1 = layer_norm_fwd(x, p["ln1_g"], p["ln1_b"], eps)
    u = rb("u", u)
    q = rb("qkv", u @ p["wq"] + p["bq"])
    k = rb("qkv", u @ p["wk"] + p["bk"])
    v = rb("qkv", u @ p["wv"] + p["bv"])
    drop = attention_dropout_factor(seed, layer, batch, seq, n_heads_total or nh, head0, nh, attn_dropout_p)
    A, P = attention_fwd(q, k, v, batch, seq, nh, head_dim, causal, rb, drop)
    Z1r = A @ p["wo"]                                                  # this rank's partial sum
    Z1 = Z1r + peers["fwd_attn"] if peers.get("fwd_attn") is not None else Z1r
    x1 = x + D1 * (Z1 + p["bo"]) * c
    v2, mu2, rstd2 = layer_norm_fwd(x1, p["ln2_g"], p["ln2_b"], eps)
    v2 = rb("v2", v2)
    pre = v2 @ p["w1"] + p["b1"]
    f = rb("f", gelu_fwd(pre, gelu_tanh))
    pre = rb("pre", pre)
    Z2r = f @ p["w2"]
    Z2 = Z2r + peers["fwd_ffn"] if peers.get("fwd_ffn") is not None else Z2r
    y = x1 + D2 * (Z2 + p["b2"]) * c
    saved = dict(x=x, u=u, mu1=mu1, rstd1=rstd1, q=q, k=k, v=v, P=P, A=A, Z1r=Z1r, Z1=Z1, x1=x1,
                 mu2=mu2, rstd2=rstd2, v2=v2, pre=pre, f=f, Z2r=Z2r, Z2=Z2, y=y, D1=D1, D2=D2, c=c,
                 batch=batch, seq=seq, head_dim=head_dim, gelu_tanh=gelu_tanh, drop=drop)
    return y, saved


def rank_layer_backward(p: dict, saved: dict, dy, *, peers: dict | None = None, bf16_sites=()):
    """Backward of one rank's share for the loss phi = <dy, y>.  `peers` may hold 'bwd_ffn' / 'bwd_attn':
    the sum of the other ranks' partial input gradients at the two backward reduction points (the
    gradient passes through each forward reduction unchanged, Eq. (1)).  Returns (dx, grads, inter)."""
    rb = _Rounder(bf16_sites)
    peers = peers or {}
    s = saved
    b, seq, d, c = s["batch"], s["seq"], s["head_dim"], s["c"]
    hp = p["wq"].shape[1]
    nh = hp // d
    g = {}
    # FFN block
    dZ2 = rb("dZ2", s["D2"] * dy * c)
    g["b2"] = dZ2.sum(dim=0)
    dx1 = dy.clone()
    dF = dZ2 @ p["w2"].t()
    g["w2"] = s["f"].t() @ dZ2
    dG = rb("dG", dF * gelu_grad(s["pre"], s["gelu_tanh"]))
    g["b1"] = dG.sum(dim=0)
    dV2r = dG @ p["w1"].t()
    g["w1"] = s["v2"].t() @ dG
    dV2 = dV2r + peers["bwd_ffn"] if peers.get("bwd_ffn") is not None else dV2r
    dln2, g["ln2_g"], g["ln2_b"] = layer_norm_bwd(dV2, s["x1"], s["mu2"], s["rstd2"], p["ln2_g"])
    dx1 = dx1 + dln2
    # attention block
    dZ1 = rb("dZ1", s["D1"] * dx1 * c)
    g["bo"] = dZ1.sum(dim=0)
    dA = rb("dA", dZ1 @ p["wo"].t())
    g["wo"] = s["A"].t() @ dZ1
    dq, dk, dv = attention_bwd(dA, s["q"], s["k"], s["v"], s["P"], b, seq, nh, d, rb, s.get("drop"))
    for n, dd in (("q", dq), ("k", dk), ("v", dv)):
        g["w" + n] = s["u"].t() @ dd
        g["b" + n] = dd.sum(dim=0)
    dUr = dq @ p["wq"].t() + dk @ p["wk"].t() + dv @ p["wv"].t()
    dU = dUr + peers["bwd_attn"] if peers.get("bwd_attn") is not None else dUr
    dln1, g["ln1_g"], g["ln1_b"] = layer_norm_bwd(dU, s["x"], s["mu1"], s["rstd1"], p["ln1_g"])
    dx = dx1 + dln1
    inter = dict(dZ2=dZ2, dG=dG, dV2r=dV2r, dV2=dV2, dx1=dx1, dZ1=dZ1, dA=dA, dq=dq, dk=dk, dv=dv,
                 dUr=dUr, dU=dU)
    return dx, g, inter


# ----------------------------------------------------------------------------------------------
# Stacked layers
# ----------------------------------------------------------------------------------------------
def to_torch(params: dict, dtype=torch.float64) -> dict:
    return {k: torch.from_numpy(np.ascontiguousarray(v)).to(dtype) for k, v in params.items()}


def model_forward_backward(layers: list, x, dy, cfg: dict, *, seed: int = 0, dtype=torch.float64,
                           bf16_sites=(), want_backward: bool = True, head0: int = 0):
    """Stack of layers (independent weights, layer l+1 reads y_l).  `layers` = list of numpy parameter
    dicts (unsharded, or one rank's slices for the rank-only computation).  Returns a dict with y, dx,
    per-layer grads and per-layer saved / intermediate tensors."""
    d = cfg["hidden"] // cfg["n_heads"]
    xt = torch.from_numpy(np.ascontiguousarray(x)).to(dtype)
    tp = [to_torch(l, dtype) for l in layers]
    saved = []
    cur = xt
    for li, p in enumerate(tp):
        cur, sv = rank_layer_forward(p, cur, batch=cfg["batch"], seq=cfg["seq"], head_dim=d,
                                     causal=bool(cfg["causal"]), dropout_p=cfg["dropout_p"], seed=seed,
                                     layer=li, bf16_sites=bf16_sites, attn_dropout_p=cfg.get("attn_dropout_p", 0.0),
                                     head0=head0, n_heads_total=cfg["n_heads"])
        saved.append(sv)
    out = dict(y=cur, saved=saved)
    if want_backward:
        g = torch.from_numpy(np.ascontiguousarray(dy)).to(dtype)
        grads, inters = [None] * len(tp), [None] * len(tp)
        for li in reversed(range(len(tp))):
            g, grads[li], inters[li] = rank_layer_backward(tp[li], saved[li], g, bf16_sites=bf16_sites)
        out.update(dx=g, grads=grads, inter=inters)
    return out
