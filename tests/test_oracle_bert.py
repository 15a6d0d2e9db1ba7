"""Pins of the post-LayerNorm (BERT-style) layer oracle: finite differences, an independent autograd derivation over
library operators, closed forms, and the Megatron shard-sum identities.  No GPU."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import bert_oracle as bo


def setup(cfg, seed=0):
    p = {k: torch.from_numpy(v).double() for k, v in si.make_layer_params(cfg, 0, seed).items()}
    x, dy = si.make_activations(cfg, seed)
    return p, torch.from_numpy(x).double(), torch.from_numpy(dy).double()


def fwd(p, x, cfg, **kw):
    return bo.rank_layer_forward(p, x, batch=cfg["batch"], seq=cfg["seq"], head_dim=cfg["hidden"] // cfg["n_heads"],
                                 causal=bool(cfg["causal"]), dropout_p=cfg["dropout_p"], seed=5, layer=1, **kw)


@pytest.mark.parametrize("causal,p_drop", [(0, 0.0), (0, 0.5), (1, 0.25)])
def test_finite_differences(causal, p_drop):
    cfg = si.small_config(causal=causal, dropout_p=p_drop)
    p, x, dy = setup(cfg)
    rng = np.random.default_rng(3)
    phi = lambda pp, xx: float((fwd(pp, xx, cfg)[0] * dy).sum())
    y, saved = fwd(p, x, cfg)
    dx, g, _ = bo.rank_layer_backward(p, saved, dy)
    eps = 1e-6
    M, h = x.shape
    for _ in range(12):
        i, j = rng.integers(M), rng.integers(h)
        xp, xm = x.clone(), x.clone()
        xp[i, j] += eps
        xm[i, j] -= eps
        fd = (phi(p, xp) - phi(p, xm)) / (2 * eps)
        assert abs(fd - float(dx[i, j])) <= 1e-6 * max(1.0, abs(fd)), ("dx", i, j)
    for name in si.PARAM_NAMES:
        flat = p[name].reshape(-1)
        for idx in rng.choice(flat.numel(), size=min(5, flat.numel()), replace=False):
            old = float(flat[idx])
            flat[idx] = old + eps
            fp_ = phi(p, x)
            flat[idx] = old - eps
            fm_ = phi(p, x)
            flat[idx] = old
            fd = (fp_ - fm_) / (2 * eps)
            assert abs(fd - float(g[name].reshape(-1)[idx])) <= 2e-6 * max(1.0, abs(fd)), (name, int(idx))


@pytest.mark.parametrize("causal,p_drop", [(0, 0.0), (1, 0.25)])
def test_against_autograd_over_library_operators(causal, p_drop):
    cfg = si.small_config(causal=causal, dropout_p=p_drop, seq=7, hidden=32, n_heads=4)
    p, x, dy = setup(cfg, seed=2)
    y, saved = fwd(p, x, cfg)
    dx, g, _ = bo.rank_layer_backward(p, saved, dy)
    pa = {k: v.clone().requires_grad_(True) for k, v in p.items()}
    xa = x.clone().requires_grad_(True)
    b, s, h, nh = cfg["batch"], cfg["seq"], cfg["hidden"], cfg["n_heads"]
    d, c = h // nh, 1.0 / (1.0 - p_drop)
    heads = lambda t: t.reshape(b, s, nh, d).transpose(1, 2)
    A = F.scaled_dot_product_attention(heads(xa @ pa["wq"] + pa["bq"]), heads(xa @ pa["wk"] + pa["bk"]), heads(xa @ pa["wv"] + pa["bv"]),
                                       is_causal=bool(causal)).transpose(1, 2).reshape(b * s, h)
    x1 = F.layer_norm(xa + saved["D1"] * (A @ pa["wo"] + pa["bo"]) * c, (h,), pa["ln1_g"], pa["ln1_b"], 1e-5)
    ya = F.layer_norm(x1 + saved["D2"] * (F.gelu(x1 @ pa["w1"] + pa["b1"], approximate="tanh") @ pa["w2"] + pa["b2"]) * c, (h,),
                      pa["ln2_g"], pa["ln2_b"], 1e-5)
    assert torch.allclose(ya, y, rtol=1e-10, atol=1e-10)
    (ya * dy).sum().backward()
    assert torch.allclose(xa.grad, dx, rtol=1e-9, atol=1e-10)
    for name in si.PARAM_NAMES:
        assert torch.allclose(pa[name].grad, g[name], rtol=1e-9, atol=1e-10), name


def test_closed_forms():
    cfg = si.small_config(causal=0)
    p, x, dy = setup(cfg)
    y, sv = fwd(p, x, cfg)
    # the output is a LayerNorm: every row of (y - beta) / gamma has mean 0 and variance 1/(1 + eps/var)
    z = (y - p["ln2_b"]) / p["ln2_g"]
    assert torch.allclose(z.mean(dim=1), torch.zeros(x.shape[0], dtype=torch.float64), atol=1e-12)
    assert torch.allclose((z * z).mean(dim=1), 1.0 - 1e-5 * sv["rstd2"].flatten() ** 2, rtol=1e-10)
    # zero row-parallel matrices and biases: both blocks add nothing, y = LN2(LN1(x))
    q = dict(p)
    for n in ("wo", "w2", "bo", "b2"):
        q[n] = torch.zeros_like(p[n])
    ref = F.layer_norm(F.layer_norm(x, (x.shape[1],), p["ln1_g"], p["ln1_b"], 1e-5), (x.shape[1],), p["ln2_g"], p["ln2_b"], 1e-5)
    assert torch.allclose(fwd(q, x, cfg)[0], ref, rtol=1e-12, atol=1e-12)
    # a gradient that is constant along a row is annihilated by the last LayerNorm when gamma is constant too
    q = dict(p)
    q["ln2_g"] = torch.full_like(p["ln2_g"], 1.5)
    y2, sv2 = fwd(q, x, cfg)
    dx, g, it = bo.rank_layer_backward(q, sv2, torch.ones_like(dy))
    assert float(it["ds2"].abs().max()) < 1e-12 and float(dx.abs().max()) < 1e-10


@pytest.mark.parametrize("t", [2, 4])
def test_megatron_shard_sum(t):
    cfg = si.small_config(hidden=32, n_heads=4, seq=5, tp=t, dropout_p=0.25, causal=0)
    pn = si.make_layer_params(cfg, 0, 0)
    x, dy = si.make_activations(cfg, 0)
    x, dy = torch.from_numpy(x).double(), torch.from_numpy(dy).double()
    full = {k: torch.from_numpy(v).double() for k, v in pn.items()}
    y, sv = fwd(full, x, cfg)
    dx, g, it = bo.rank_layer_backward(full, sv, dy)
    shards = [{k: torch.from_numpy(v).double() for k, v in si.shard_layer_params(pn, cfg, r).items()} for r in range(t)]
    z1 = [fwd(s, x, cfg)[1]["Z1r"] for s in shards]
    assert torch.allclose(sum(z1), sv["Z1"], rtol=1e-11, atol=1e-12)
    hp, fp = cfg["hidden"] // t, 4 * cfg["hidden"] // t
    for r in range(t):
        peers = {"fwd_attn": sv["Z1"] - z1[r]}
        _, svr = fwd(shards[r], x, cfg, peers=peers)
        peers["fwd_ffn"] = sv["Z2"] - svr["Z2r"]
        yr, svr = fwd(shards[r], x, cfg, peers=peers)
        assert torch.allclose(yr, y, rtol=1e-11, atol=1e-12)
        _, _, itr = bo.rank_layer_backward(shards[r], svr, dy)
        bp = {"bwd_ffn": it["dV2"] - itr["dV2r"]}
        _, _, itr = bo.rank_layer_backward(shards[r], svr, dy, peers=bp)
        bp["bwd_attn"] = it["dU"] - itr["dUr"]
        dxr, gr, _ = bo.rank_layer_backward(shards[r], svr, dy, peers=bp)
        assert torch.allclose(dxr, dx, rtol=1e-10, atol=1e-11)
        a, f = slice(r * hp, (r + 1) * hp), slice(r * fp, (r + 1) * fp)
        for n in ("wq", "wk", "wv"):
            assert torch.allclose(gr[n], g[n][:, a], rtol=1e-10, atol=1e-11), n
        for n in ("bq", "bk", "bv"):
            assert torch.allclose(gr[n], g[n][a], rtol=1e-10, atol=1e-11), n
        assert torch.allclose(gr["wo"], g["wo"][a, :], rtol=1e-10, atol=1e-11)
        assert torch.allclose(gr["w1"], g["w1"][:, f], rtol=1e-10, atol=1e-11) and torch.allclose(gr["b1"], g["b1"][f], rtol=1e-10, atol=1e-11)
        assert torch.allclose(gr["w2"], g["w2"][f, :], rtol=1e-10, atol=1e-11)
        for n in ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "bo", "b2"):
            assert torch.allclose(gr[n], g[n], rtol=1e-10, atol=1e-11), n
