"""Pins of the LLaMA-style layer oracle: finite differences, an independent autograd derivation over library
operators (rms_norm, scaled_dot_product_attention, silu) with the rotary embedding written as a complex product,
closed forms and invariants of the rotation, and the Megatron shard-sum identities.  No GPU."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import synth_inputs as si
from oracle import llama_oracle as ll

NAMES = ("ln1_g", "wq", "wk", "wv", "wo", "ln2_g", "wg", "wu", "w2")


def small(**over):
    c = dict(arch="llama", hidden=16, n_heads=2, seq=6, batch=2, tp=1, n_sub=1, n_layers=1, causal=1, dropout_p=0.0, ffn_hidden=24,
             rope_theta=10000.0, w_sigma=0.25)
    c.update(over)
    return c


def setup(cfg, seed=0):
    p = {k: torch.from_numpy(v).double() for k, v in si.make_llama_layer_params(cfg, 0, seed).items()}
    x, dy = si.make_activations(cfg, seed)
    return p, torch.from_numpy(x).double(), torch.from_numpy(dy).double()


def fwd(p, x, cfg, **kw):
    return ll.rank_layer_forward(p, x, batch=cfg["batch"], seq=cfg["seq"], head_dim=cfg["hidden"] // cfg["n_heads"],
                                 causal=bool(cfg["causal"]), dropout_p=cfg["dropout_p"], seed=5, layer=1, theta=cfg["rope_theta"], **kw)


@pytest.mark.parametrize("causal,p_drop", [(1, 0.0), (0, 0.5), (1, 0.5)])
def test_finite_differences(causal, p_drop):
    cfg = small(causal=causal, dropout_p=p_drop)
    p, x, dy = setup(cfg)
    rng = np.random.default_rng(3)
    phi = lambda pp, xx: float((fwd(pp, xx, cfg)[0] * dy).sum())
    y, saved = fwd(p, x, cfg)
    dx, g, _ = ll.rank_layer_backward(p, saved, dy)
    eps = 1e-6
    M, h = x.shape
    for _ in range(12):
        i, j = rng.integers(M), rng.integers(h)
        xp, xm = x.clone(), x.clone()
        xp[i, j] += eps
        xm[i, j] -= eps
        fd = (phi(p, xp) - phi(p, xm)) / (2 * eps)
        assert abs(fd - float(dx[i, j])) <= 1e-6 * max(1.0, abs(fd)), ("dx", i, j)
    for name in NAMES:
        flat = p[name].reshape(-1)
        for idx in rng.choice(flat.numel(), size=min(6, flat.numel()), replace=False):
            old = float(flat[idx])
            flat[idx] = old + eps
            fp_ = phi(p, x)
            flat[idx] = old - eps
            fm_ = phi(p, x)
            flat[idx] = old
            fd = (fp_ - fm_) / (2 * eps)
            assert abs(fd - float(g[name].reshape(-1)[idx])) <= 2e-6 * max(1.0, abs(fd)), (name, int(idx))


def library_layer(p, x, cfg, D1, D2):
    """The same layer through library operators and a different formulation of the rotation: a head's pair
    (x_i, x_{i+d/2}) is the complex number x_i + i x_{i+d/2}, multiplied by exp(i * pos * theta^(-2i/d))."""
    b, s, h, nh = cfg["batch"], cfg["seq"], cfg["hidden"], p["wq"].shape[1] // (cfg["hidden"] // cfg["n_heads"])
    d = cfg["hidden"] // cfg["n_heads"]
    c = 1.0 / (1.0 - cfg["dropout_p"])

    def rot(t):
        t = t.reshape(b, s, nh, d)
        z = torch.complex(t[..., : d // 2], t[..., d // 2:])
        freq = cfg["rope_theta"] ** (-torch.arange(0, d, 2, dtype=torch.float64) / d)
        ph = torch.polar(torch.ones(s, d // 2, dtype=torch.float64), torch.arange(s, dtype=torch.float64)[:, None] * freq[None, :])
        z = z * ph[None, :, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    u = F.rms_norm(x, (h,), p["ln1_g"], eps=1e-5)
    q, k = rot(u @ p["wq"]).transpose(1, 2), rot(u @ p["wk"]).transpose(1, 2)
    v = (u @ p["wv"]).reshape(b, s, nh, d).transpose(1, 2)
    A = F.scaled_dot_product_attention(q, k, v, is_causal=bool(cfg["causal"])).transpose(1, 2).reshape(b * s, nh * d)
    x1 = x + D1 * (A @ p["wo"]) * c
    v2 = F.rms_norm(x1, (h,), p["ln2_g"], eps=1e-5)
    return x1 + D2 * ((F.silu(v2 @ p["wg"]) * (v2 @ p["wu"])) @ p["w2"]) * c


@pytest.mark.parametrize("causal,p_drop", [(1, 0.0), (0, 0.25)])
def test_against_autograd_over_library_operators(causal, p_drop):
    cfg = small(causal=causal, dropout_p=p_drop, seq=9, hidden=32, n_heads=4, ffn_hidden=40)
    p, x, dy = setup(cfg, seed=2)
    y, saved = fwd(p, x, cfg)
    dx, g, _ = ll.rank_layer_backward(p, saved, dy)
    pa = {k: v.clone().requires_grad_(True) for k, v in p.items()}
    xa = x.clone().requires_grad_(True)
    ya = library_layer(pa, xa, cfg, saved["D1"], saved["D2"])
    assert torch.allclose(ya, y, rtol=1e-10, atol=1e-10)
    (ya * dy).sum().backward()
    assert torch.allclose(xa.grad, dx, rtol=1e-9, atol=1e-10)
    for name in NAMES:
        assert torch.allclose(pa[name].grad, g[name], rtol=1e-9, atol=1e-10), name


def test_rotary_closed_forms_and_invariants():
    b, s, nh, d = 2, 7, 3, 8
    g = torch.Generator().manual_seed(1)
    q = torch.randn(b * s, nh * d, dtype=torch.float64, generator=g)
    k = torch.randn(b * s, nh * d, dtype=torch.float64, generator=g)
    rq, rk = ll.rope_apply(q, b, s, d, 10000.0), ll.rope_apply(k, b, s, d, 10000.0)
    # position 0 is not rotated; a rotation keeps every pair's length; the inverse undoes it
    assert torch.equal(rq.reshape(b, s, -1)[:, 0], q.reshape(b, s, -1)[:, 0])
    n2 = lambda t: (t.reshape(b, s, nh, 2, d // 2) ** 2).sum(dim=3)
    assert torch.allclose(n2(rq), n2(q), rtol=1e-13)
    assert torch.allclose(ll.rope_apply(rq, b, s, d, 10000.0, inverse=True), q, rtol=1e-12, atol=1e-13)
    # hand value: pair 0 of head 0 at position 3 turns by 3 rad (theta^0 = 1); pair 1 by 3 * 10000^(-2/8)
    x = q.reshape(b, s, nh, d)[1, 3, 0]
    y = rq.reshape(b, s, nh, d)[1, 3, 0]
    import math
    assert float(y[0]) == pytest.approx(float(x[0]) * math.cos(3.0) - float(x[4]) * math.sin(3.0), rel=1e-12)
    assert float(y[4]) == pytest.approx(float(x[4]) * math.cos(3.0) + float(x[0]) * math.sin(3.0), rel=1e-12)
    a1 = 3.0 * 10000.0 ** (-2.0 / 8.0)
    assert float(y[1]) == pytest.approx(float(x[1]) * math.cos(a1) - float(x[5]) * math.sin(a1), rel=1e-12)
    # relative position: the score of a query at position m against a key at position n depends on m - n only, so
    # moving the same content two positions later leaves it unchanged
    qq, kk = q.reshape(b, s, nh, d), k.reshape(b, s, nh, d)
    q2, k2 = qq.clone(), kk.clone()
    q2[:, 5], k2[:, 3] = qq[:, 3], kk[:, 1]
    r2q, r2k = ll.rope_apply(q2.reshape(b * s, -1), b, s, d, 10000.0), ll.rope_apply(k2.reshape(b * s, -1), b, s, d, 10000.0)
    s_a = (rq.reshape(b, s, nh, d)[:, 3] * rk.reshape(b, s, nh, d)[:, 1]).sum(-1)
    s_b = (r2q.reshape(b, s, nh, d)[:, 5] * r2k.reshape(b, s, nh, d)[:, 3]).sum(-1)
    assert torch.allclose(s_a, s_b, rtol=1e-11, atol=1e-12)


def test_norm_and_activation_closed_forms():
    x = torch.tensor([[3.0, -4.0, 0.0, 0.0]], dtype=torch.float64)
    y, rstd = ll.rms_norm_fwd(x, torch.tensor([1.0, 2.0, 3.0, 4.0], dtype=torch.float64), 0.0)
    assert float(rstd) == pytest.approx(1.0 / 2.5) and torch.allclose(y, torch.tensor([[1.2, -3.2, 0.0, 0.0]], dtype=torch.float64))
    z = torch.tensor([0.0, 1.0, -2.0], dtype=torch.float64)
    assert torch.allclose(ll.silu(z), z / (1 + torch.exp(-z)))
    assert float(ll.silu_grad(torch.tensor(0.0, dtype=torch.float64))) == 0.5
    e = 1e-6
    assert torch.allclose(ll.silu_grad(z), (ll.silu(z + e) - ll.silu(z - e)) / (2 * e), rtol=1e-8)
    # zero weight matrices: the layer is the identity on the residual stream
    cfg = small()
    p, xx, _ = setup(cfg)
    for n in ("wo", "w2"):
        p[n] = torch.zeros_like(p[n])
    assert torch.equal(fwd(p, xx, cfg)[0], xx)


@pytest.mark.parametrize("t", [2, 4])
def test_megatron_shard_sum(t):
    """Sum over ranks of the partial results = the unsharded ones; with the peers' sums every rank reproduces y and dx;
    gradient shards are slices of the unsharded gradients (Sec. II; Sec. IV-B Eq. (1))."""
    cfg = small(hidden=32, n_heads=4, seq=5, ffn_hidden=48, tp=t, dropout_p=0.25)
    pn = si.make_llama_layer_params(cfg, 0, 0)
    x, dy = si.make_activations(cfg, 0)
    x, dy = torch.from_numpy(x).double(), torch.from_numpy(dy).double()
    full = {k: torch.from_numpy(v).double() for k, v in pn.items()}
    y, sv = fwd(full, x, cfg)
    dx, g, it = ll.rank_layer_backward(full, sv, dy)
    shards = [{k: torch.from_numpy(v).double() for k, v in si.shard_llama_layer_params(pn, cfg, r).items()} for r in range(t)]
    outs = [fwd(s, x, cfg, peers={"fwd_attn": None, "fwd_ffn": None}) for s in shards]
    # forward reduction points: the partial sums are linear in the rank's slice only if the inputs agree, so feed the true sums
    z1 = [o[1]["Z1r"] for o in outs]
    assert torch.allclose(sum(z1), sv["Z1"], rtol=1e-11, atol=1e-12)
    hp, fp = cfg["hidden"] // t, cfg["ffn_hidden"] // t
    for r in range(t):
        peers = {"fwd_attn": sv["Z1"] - z1[r]}
        yr, svr = fwd(shards[r], x, cfg, peers={**peers, "fwd_ffn": None})
        peers["fwd_ffn"] = sv["Z2"] - svr["Z2r"]
        yr, svr = fwd(shards[r], x, cfg, peers=peers)
        assert torch.allclose(yr, y, rtol=1e-11, atol=1e-12)
        dxr, gr, itr = ll.rank_layer_backward(shards[r], svr, dy)
        bp = {"bwd_ffn": it["dV2"] - itr["dV2r"]}
        dxr, gr, itr = ll.rank_layer_backward(shards[r], svr, dy, peers=bp)
        bp["bwd_attn"] = it["dU"] - itr["dUr"]
        dxr, gr, itr = ll.rank_layer_backward(shards[r], svr, dy, peers=bp)
        assert torch.allclose(dxr, dx, rtol=1e-10, atol=1e-11)
        a, f = slice(r * hp, (r + 1) * hp), slice(r * fp, (r + 1) * fp)
        for n in ("wq", "wk", "wv"):
            assert torch.allclose(gr[n], g[n][:, a], rtol=1e-10, atol=1e-11), n
        assert torch.allclose(gr["wo"], g["wo"][a, :], rtol=1e-10, atol=1e-11)
        for n in ("wg", "wu"):
            assert torch.allclose(gr[n], g[n][:, f], rtol=1e-10, atol=1e-11), n
        assert torch.allclose(gr["w2"], g["w2"][f, :], rtol=1e-10, atol=1e-11)
        for n in ("ln1_g", "ln2_g"):
            assert torch.allclose(gr[n], g[n], rtol=1e-10, atol=1e-11), n
