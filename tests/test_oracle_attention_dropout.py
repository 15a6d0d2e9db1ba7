"""Pins of the attention-probability dropout of the layer oracle: the mask's counter / byte layout by brute force over
single Philox calls (the generator itself is pinned by known-answer vectors in test_oracle_philox.py), invariance to the
partition, finite differences and an autograd derivation over library softmax with the mask as a given factor."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import layer_oracle as lo


def test_mask_layout_by_single_calls():
    seed, layer, batch, seq, nht, head0, nhl, p = 0x1234567890ABCDEF, 3, 2, 11, 8, 4, 2, 0.3
    f = lo.attention_dropout_factor(seed, layer, batch, seq, nht, head0, nhl, p)
    T = lo.attention_dropout_threshold(p)
    assert T == 77 and f.shape == (batch, nhl, seq, seq)
    rng = np.random.default_rng(0)
    for _ in range(60):
        b, hl, q, k = rng.integers(batch), rng.integers(nhl), rng.integers(seq), rng.integers(seq)
        w = lo.philox4x32_10([k // 4], [q // 4], [b * nht + head0 + hl], [layer | 0x80000000], seed & 0xFFFFFFFF, seed >> 32)
        byte = (int(w[q % 4][0]) >> (8 * (k % 4))) & 0xFF
        want = 256.0 / (256.0 - T) if byte >= T else 0.0
        assert float(f[b, hl, q, k]) == want, (b, hl, q, k)
    # the rate is the quantised one and the factor is unbiased
    big = lo.attention_dropout_factor(1, 0, 4, 128, 4, 0, 4, 0.1)
    assert abs(float((big > 0).double().mean()) - (1 - 26 / 256)) < 3e-3 and abs(float(big.mean()) - 1.0) < 4e-3
    assert lo.attention_dropout_factor(1, 0, 1, 8, 1, 0, 1, 0.001) is None          # rounds to rate 0


def test_mask_does_not_depend_on_the_partition():
    full = lo.attention_dropout_factor(5, 2, 3, 20, 8, 0, 8, 0.25)
    for t in (2, 4):
        for r in range(t):
            part = lo.attention_dropout_factor(5, 2, 3, 20, 8, r * (8 // t), 8 // t, 0.25)
            assert torch.equal(part, full[:, r * (8 // t):(r + 1) * (8 // t)])


def _fwd(p, x, cfg, **kw):
    return lo.rank_layer_forward(p, x, batch=cfg["batch"], seq=cfg["seq"], head_dim=cfg["hidden"] // cfg["n_heads"], causal=bool(cfg["causal"]),
                                 dropout_p=cfg["dropout_p"], seed=5, layer=1, attn_dropout_p=cfg["attn_dropout_p"], **kw)


@pytest.mark.parametrize("causal", [0, 1])
def test_finite_differences_with_attention_dropout(causal):
    cfg = si.small_config(causal=causal, dropout_p=0.25, attn_dropout_p=0.4, seq=6)
    p = lo.to_torch(si.make_layer_params(cfg, 0, 0))
    x, dy = (torch.from_numpy(a).double() for a in si.make_activations(cfg, 0))
    phi = lambda pp, xx: float((_fwd(pp, xx, cfg)[0] * dy).sum())
    y, saved = _fwd(p, x, cfg)
    assert saved["drop"] is not None and float((saved["drop"] == 0).double().mean()) > 0.2
    dx, g, _ = lo.rank_layer_backward(p, saved, dy)
    rng = np.random.default_rng(1)
    eps = 1e-6
    for _ in range(10):
        i, j = rng.integers(x.shape[0]), rng.integers(x.shape[1])
        xp, xm = x.clone(), x.clone()
        xp[i, j] += eps
        xm[i, j] -= eps
        fd = (phi(p, xp) - phi(p, xm)) / (2 * eps)
        assert abs(fd - float(dx[i, j])) <= 1e-6 * max(1.0, abs(fd))
    for name in ("wq", "wk", "wv", "bq", "bv", "wo", "ln1_g"):
        flat = p[name].reshape(-1)
        for idx in rng.choice(flat.numel(), size=5, replace=False):
            old = float(flat[idx])
            flat[idx] = old + eps
            a = phi(p, x)
            flat[idx] = old - eps
            b = phi(p, x)
            flat[idx] = old
            fd = (a - b) / (2 * eps)
            assert abs(fd - float(g[name].reshape(-1)[idx])) <= 2e-6 * max(1.0, abs(fd)), (name, int(idx))


def test_attention_operator_against_autograd_over_library_softmax():
    b, s, nh, d = 2, 9, 3, 8
    g = torch.Generator().manual_seed(3)
    q, k, v, dA = (torch.randn(b * s, nh * d, dtype=torch.float64, generator=g) for _ in range(4))
    drop = lo.attention_dropout_factor(9, 0, b, s, nh, 0, nh, 0.3)
    A, P = lo.attention_fwd(q, k, v, b, s, nh, d, True, drop=drop)
    dq, dk, dv = lo.attention_bwd(dA, q, k, v, P, b, s, nh, d, drop=drop)
    qa, ka, va = (t.clone().requires_grad_(True) for t in (q, k, v))
    heads = lambda t: t.reshape(b, s, nh, d).transpose(1, 2)
    S = heads(qa) @ heads(ka).transpose(2, 3) / math.sqrt(d)
    S = S.masked_fill(torch.ones(s, s, dtype=torch.bool).triu(1), float("-inf"))
    Aa = ((torch.softmax(S, dim=3) * drop) @ heads(va)).transpose(1, 2).reshape(b * s, nh * d)
    assert torch.allclose(Aa, A, rtol=1e-12, atol=1e-12)
    (Aa * dA).sum().backward()
    for got, ref in ((dq, qa.grad), (dk, ka.grad), (dv, va.grad)):
        assert torch.allclose(got, ref, rtol=1e-10, atol=1e-11)
    # rate 0 is the plain operator
    A0, _ = lo.attention_fwd(q, k, v, b, s, nh, d, True)
    assert torch.equal(lo.attention_fwd(q, k, v, b, s, nh, d, True, drop=None)[0], A0)
