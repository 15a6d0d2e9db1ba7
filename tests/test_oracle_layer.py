"""Pins for the layer oracle: finite differences, an independent autograd derivation over library
operators, closed forms, and the Megatron shard-sum identities (Sec. II TMP; Sec. IV-B Eq. (1))."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import layer_oracle as lo

torch.manual_seed(0)


def _setup(cfg, seed=0, perturb_bias=True):
    p = si.make_layer_params(cfg, 0, seed)
    x, dy = si.make_activations(cfg, seed)
    return p, x, dy


def _fwd(p, x, cfg, **kw):
    d = cfg["hidden"] // cfg["n_heads"]
    return lo.rank_layer_forward(p, x, batch=cfg["batch"], seq=cfg["seq"], head_dim=d,
                                 causal=bool(cfg["causal"]), dropout_p=cfg["dropout_p"], seed=5, layer=1, **kw)


# ------------------------------------------------------------------ finite differences (fp64)
@pytest.mark.parametrize("causal,p_drop,with_peers", [(1, 0.0, False), (0, 0.5, False), (1, 0.5, True)])
def test_finite_differences(causal, p_drop, with_peers):
    cfg = si.small_config(causal=causal, dropout_p=p_drop)
    pn, x, dy = _setup(cfg)
    p = lo.to_torch(pn)
    xt, dyt = torch.from_numpy(x).double(), torch.from_numpy(dy).double()
    rng = np.random.default_rng(3)
    M, h = x.shape
    peers = None
    if with_peers:
        peers = {k: torch.from_numpy(rng.standard_normal((M, h))) for k in ("fwd_attn", "fwd_ffn", "bwd_ffn", "bwd_attn")}

    def phi(pp, xx):
        y, _ = _fwd(pp, xx, cfg, peers=peers)
        return float((y * dyt).sum())

    y, saved = _fwd(p, xt, cfg, peers=peers)
    # backward peers are *gradient* inputs; for the FD check of phi they must be absent
    dx, g, _ = lo.rank_layer_backward(p, saved, dyt)
    eps = 1e-6
    # input gradient
    for _ in range(12):
        i, j = rng.integers(M), rng.integers(h)
        xp, xm = xt.clone(), xt.clone()
        xp[i, j] += eps
        xm[i, j] -= eps
        fd = (phi(p, xp) - phi(p, xm)) / (2 * eps)
        assert abs(fd - float(dx[i, j])) <= 1e-6 * max(1.0, abs(fd)), ("dx", i, j)
    # every parameter gradient
    for name in si.PARAM_NAMES:
        t = p[name]
        flat = t.reshape(-1)
        for idx in rng.choice(flat.numel(), size=min(6, flat.numel()), replace=False):
            old = float(flat[idx])
            flat[idx] = old + eps
            fp = phi(p, xt)
            flat[idx] = old - eps
            fm = phi(p, xt)
            flat[idx] = old
            fd = (fp - fm) / (2 * eps)
            an = float(g[name].reshape(-1)[idx])
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(fd)), (name, int(idx), fd, an)


def test_backward_peer_sums_enter_linearly():
    # dV2 = dV2_r + peer, dU = dU_r + peer: with a peer, dx changes by LN'(peer) exactly (LN' is linear in dy)
    cfg = si.small_config()
    pn, x, dy = _setup(cfg)
    p = lo.to_torch(pn)
    xt, dyt = torch.from_numpy(x).double(), torch.from_numpy(dy).double()
    y, saved = _fwd(p, xt, cfg)
    dx0, _, _ = lo.rank_layer_backward(p, saved, dyt)
    peer = torch.from_numpy(np.random.default_rng(1).standard_normal(x.shape))
    dx1, _, it = lo.rank_layer_backward(p, saved, dyt, peers={"bwd_attn": peer})
    extra, _, _ = lo.layer_norm_bwd(peer, saved["x"], saved["mu1"], saved["rstd1"], p["ln1_g"])
    assert torch.allclose(dx1 - dx0, extra, atol=1e-12)
    assert torch.allclose(it["dU"], it["dUr"] + peer)


# ------------------------------------------------------------------ independent autograd derivation
def _autograd_layer(p, x, cfg, D1, D2):
    h = cfg["hidden"]
    nh, b, s = cfg["n_heads"], cfg["batch"], cfg["seq"]
    d = h // nh
    c = 1.0 / (1.0 - cfg["dropout_p"])
    u = F.layer_norm(x, (h,), p["ln1_g"], p["ln1_b"], 1e-5)
    q, k, v = (F.linear(u, p["w" + n].t(), p["b" + n]).reshape(b, s, nh, d).transpose(1, 2) for n in "qkv")
    a = F.scaled_dot_product_attention(q, k, v, is_causal=bool(cfg["causal"]))
    a = a.transpose(1, 2).reshape(b * s, h)
    x1 = x + D1 * F.linear(a, p["wo"].t(), p["bo"]) * c
    v2 = F.layer_norm(x1, (h,), p["ln2_g"], p["ln2_b"], 1e-5)
    f = F.gelu(F.linear(v2, p["w1"].t(), p["b1"]), approximate="tanh")
    return x1 + D2 * F.linear(f, p["w2"].t(), p["b2"]) * c


@pytest.mark.parametrize("causal,p_drop", [(1, 0.1), (0, 0.0)])
def test_against_autograd_of_library_ops(causal, p_drop):
    cfg = dict(hidden=64, n_heads=4, seq=24, batch=3, tp=1, n_sub=1, n_layers=1, causal=causal,
               dropout_p=p_drop, w_sigma=0.1)
    pn, x, dy = _setup(cfg)
    p = lo.to_torch(pn)
    xt, dyt = torch.from_numpy(x).double(), torch.from_numpy(dy).double()
    y, saved = _fwd(p, xt, cfg)
    dx, g, _ = lo.rank_layer_backward(p, saved, dyt)
    pa = {k: v.clone().requires_grad_(True) for k, v in p.items()}
    xa = xt.clone().requires_grad_(True)
    ya = _autograd_layer(pa, xa, cfg, saved["D1"], saved["D2"])
    (ya * dyt).sum().backward()
    assert torch.allclose(y, ya.detach(), rtol=1e-10, atol=1e-10)
    assert torch.allclose(dx, xa.grad, rtol=1e-9, atol=1e-10)
    for name in si.PARAM_NAMES:
        assert torch.allclose(g[name], pa[name].grad, rtol=1e-9, atol=1e-10), name


# ------------------------------------------------------------------ closed forms
def test_closed_forms():
    cfg = dict(hidden=32, n_heads=2, seq=6, batch=2, tp=1, n_sub=1, n_layers=1, causal=1, dropout_p=0.0, w_sigma=0.3)
    pn, x, dy = _setup(cfg)
    p = lo.to_torch(pn)
    xt = torch.from_numpy(x).double()
    y, sv = _fwd(p, xt, cfg)
    b, s, h = cfg["batch"], cfg["seq"], cfg["hidden"]
    # softmax rows sum to one, causal: nothing above the diagonal
    assert torch.allclose(sv["P"].sum(dim=3), torch.ones(b, 2, s, dtype=torch.float64))
    assert float(sv["P"].triu(1).abs().max()) == 0.0
    # first token of every sequence sees only itself: a_0 = v_0
    A, v = sv["A"].reshape(b, s, h), sv["v"].reshape(b, s, h)
    assert torch.allclose(A[:, 0], v[:, 0], atol=1e-14)
    # LayerNorm with gamma=1, beta=0: zero mean, variance var/(var+eps)
    z, mu, rstd = lo.layer_norm_fwd(xt, torch.ones(h, dtype=torch.float64), torch.zeros(h, dtype=torch.float64), 1e-5)
    assert float(z.mean(dim=1).abs().max()) < 1e-14
    var = xt.var(dim=1, unbiased=False)
    assert torch.allclose((z ** 2).mean(dim=1), var / (var + 1e-5))
    # Wq = 0, bq = 0  =>  uniform attention over the visible prefix: A_i = mean_{j<=i} v_j
    p0 = dict(p)
    p0["wq"], p0["bq"] = torch.zeros_like(p["wq"]), torch.zeros_like(p["bq"])
    _, sv0 = _fwd(p0, xt, cfg)
    v0 = sv0["v"].reshape(b, s, h)
    pref = torch.cumsum(v0, dim=1) / torch.arange(1, s + 1, dtype=torch.float64)[None, :, None]
    assert torch.allclose(sv0["A"].reshape(b, s, h), pref, atol=1e-13)
    # all matrices zero => y = x + bo + b2 (dropout off)
    pz = {k: (torch.zeros_like(t) if k in ("wq", "wk", "wv", "wo", "w1", "w2") else t) for k, t in p.items()}
    pz["b1"] = torch.zeros_like(p["b1"])
    yz, _ = _fwd(pz, xt, cfg)
    assert torch.allclose(yz, xt + p["bo"] + p["b2"], atol=1e-14)
    # GeLU values: gelu(0) = 0, gelu'(0) = 1/2, tanh form close to the erf form
    t = torch.tensor([0.0, 1.0, -2.5, 3.0], dtype=torch.float64)
    assert float(lo.gelu_fwd(t)[0]) == 0.0 and float(lo.gelu_grad(t)[0]) == 0.5
    assert torch.allclose(lo.gelu_fwd(t), lo.gelu_fwd(t, tanh_form=False), atol=2e-3)
    assert abs(float(lo.gelu_fwd(t)[1]) - 0.841192) < 1e-6    # 0.5*(1+tanh(sqrt(2/pi)*1.044715))


def test_seq_one_attention_is_identity_on_v():
    cfg = dict(hidden=16, n_heads=2, seq=1, batch=5, tp=1, n_sub=1, n_layers=1, causal=0, dropout_p=0.0, w_sigma=0.3)
    pn, x, _ = _setup(cfg)
    _, sv = _fwd(lo.to_torch(pn), torch.from_numpy(x).double(), cfg)
    assert torch.allclose(sv["A"], sv["v"], atol=1e-15)


def test_dropout_scales_kept_values():
    cfg = si.small_config(dropout_p=0.5)
    pn, x, _ = _setup(cfg)
    p = lo.to_torch(pn)
    xt = torch.from_numpy(x).double()
    _, sv = _fwd(p, xt, cfg)
    kept = sv["D1"].bool()
    want = xt + 2.0 * (sv["Z1"] + p["bo"])
    assert torch.allclose(sv["x1"][kept], want[kept]) and torch.equal(sv["x1"][~kept], xt[~kept])


# ------------------------------------------------------------------ tensor-model-parallel structure
@pytest.mark.parametrize("t", [1, 2, 4])
def test_rank_partials_sum_to_the_unsharded_layer(t):
    cfg = dict(hidden=64, n_heads=4, seq=8, batch=2, tp=t, n_sub=1, n_layers=1, causal=1, dropout_p=0.25, w_sigma=0.1)
    pn, x, dy = _setup(cfg)
    xt, dyt = torch.from_numpy(x).double(), torch.from_numpy(dy).double()
    full = lo.to_torch(pn)
    y, sv = _fwd(full, xt, cfg)
    dx, g, it = lo.rank_layer_backward(full, sv, dyt)
    ranks = [lo.to_torch(si.shard_layer_params(pn, cfg, r)) for r in range(t)]
    # lock-step emulation: forward to the first reduction point with no peers gives each partial
    part = [_fwd(rp, xt, cfg)[1] for rp in ranks]
    Z1 = sum(s_["Z1r"] for s_ in part)
    assert torch.allclose(Z1, sv["Z1"], atol=1e-12)
    part = [_fwd(rp, xt, cfg, peers={"fwd_attn": Z1 - part[r]["Z1r"]})[1] for r, rp in enumerate(ranks)]
    Z2 = sum(s_["Z2r"] for s_ in part)
    assert torch.allclose(Z2, sv["Z2"], atol=1e-12)
    outs = [_fwd(rp, xt, cfg, peers={"fwd_attn": Z1 - part[r]["Z1r"], "fwd_ffn": Z2 - part[r]["Z2r"]})
            for r, rp in enumerate(ranks)]
    for yr, _ in outs:
        assert torch.allclose(yr, y, atol=1e-12)        # every rank holds the full output
    # backward: same lock-step on the two backward reduction points
    b0 = [lo.rank_layer_backward(rp, outs[r][1], dyt)[2] for r, rp in enumerate(ranks)]
    dV2 = sum(i_["dV2r"] for i_ in b0)
    assert torch.allclose(dV2, it["dV2"], atol=1e-12)
    b1 = [lo.rank_layer_backward(rp, outs[r][1], dyt, peers={"bwd_ffn": dV2 - b0[r]["dV2r"]})[2]
          for r, rp in enumerate(ranks)]
    dU = sum(i_["dUr"] for i_ in b1)
    assert torch.allclose(dU, it["dU"], atol=1e-12)
    hp, fp = 64 // t, 256 // t
    for r, rp in enumerate(ranks):
        dxr, gr, _ = lo.rank_layer_backward(rp, outs[r][1], dyt,
                                            peers={"bwd_ffn": dV2 - b0[r]["dV2r"], "bwd_attn": dU - b1[r]["dUr"]})
        assert torch.allclose(dxr, dx, atol=1e-12)
        a, f = slice(r * hp, (r + 1) * hp), slice(r * fp, (r + 1) * fp)
        for n in ("wq", "wk", "wv"):
            assert torch.allclose(gr[n], g[n][:, a], atol=1e-12)
        for n in ("bq", "bk", "bv"):
            assert torch.allclose(gr[n], g[n][a], atol=1e-12)
        assert torch.allclose(gr["wo"], g["wo"][a, :], atol=1e-12)
        assert torch.allclose(gr["w1"], g["w1"][:, f], atol=1e-12)
        assert torch.allclose(gr["b1"], g["b1"][f], atol=1e-12)
        assert torch.allclose(gr["w2"], g["w2"][f, :], atol=1e-12)
        for n in ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "bo", "b2"):     # replicated parameters
            assert torch.allclose(gr[n], g[n], atol=1e-12)


def test_stacked_layers_chain():
    cfg = dict(hidden=32, n_heads=2, seq=4, batch=2, tp=1, n_sub=1, n_layers=2, causal=1, dropout_p=0.1, w_sigma=0.1)
    layers = [si.make_layer_params(cfg, l, 0) for l in range(2)]
    x, dy = si.make_activations(cfg, 0)
    out = lo.model_forward_backward(layers, x, dy, cfg, seed=9)
    assert out["saved"][1]["x"] is out["saved"][0]["y"]
    # different Philox layer word => different masks per layer
    assert not torch.equal(out["saved"][0]["D1"], out["saved"][1]["D1"])
    # FD through both layers on one input element
    xt = torch.from_numpy(x).double()
    eps = 1e-6

    def phi(xx):
        o = lo.model_forward_backward(layers, xx.numpy(), dy, cfg, seed=9, want_backward=False)
        return float((o["y"] * torch.from_numpy(dy).double()).sum())
    xp, xm = xt.clone(), xt.clone()
    xp[3, 7] += eps
    xm[3, 7] -= eps
    fd = (phi(xp) - phi(xm)) / (2 * eps)
    assert abs(fd - float(out["dx"][3, 7])) < 1e-6 * max(1.0, abs(fd))
