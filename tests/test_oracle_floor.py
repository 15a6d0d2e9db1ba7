"""Pins of the storage-format floor tool of the oracle (the `bf16_sites` option of oracle/layer_oracle.py): the GPU
parity gate calls a tensor FORMAT-LIMITED only relative to this tool, so what it does must be fixed by something other
than itself.  On a tiny layer, with ONE site switched on at a time:
  * the rounding is round-to-nearest-even to 8 significant bits, checked on the bit pattern;
  * the tensor at the site is exactly the bf16 rounding of the unrounded run's tensor, and everything upstream of the
    site is bit-identical to the unrounded run (the rounding sits on that tensor and nowhere before it);
  * the immediate consumers of the site see the rounded tensor: each is recomputed here by hand from the rounded
    tensor with plain matmul / softmax, one formula per site.
And the list of sites is the list of tensors the library stores as bf16 (workspace plan through the C ABI, host only)
plus the two MFMA operands that never leave registers (P, dS)."""
import math

import numpy as np
import pytest
import torch

from oracle import layer_oracle as lo

CFG = dict(hidden=32, n_heads=4, seq=8, batch=2, tp=1, n_sub=1, n_layers=1, causal=1, dropout_p=0.25, w_sigma=0.3)


def bf16_by_hand(t):
    """Round-to-nearest-even of fp32 values to 8 significant bits, on the bit pattern."""
    u = t.to(torch.float32).contiguous().numpy().view(np.uint32).astype(np.uint64)
    r = ((u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))) >> np.uint64(16)) << np.uint64(16)
    return torch.from_numpy((r & np.uint64(0xFFFFFFFF)).astype(np.uint32).view(np.float32).copy()).reshape(t.shape)


def test_rounding_is_nearest_even_to_eight_bits():
    x = torch.tensor([1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8), 0.1, 65504.0, 0.0])
    want = torch.tensor([1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -1.0, 0.10009765625, 65536.0, 0.0])
    assert torch.equal(lo._bf16(x), want)
    g = torch.Generator().manual_seed(1)
    r = torch.randn(4096, generator=g) * torch.exp(4 * torch.randn(4096, generator=g))
    assert torch.equal(lo._bf16(r), bf16_by_hand(r))
    assert torch.equal(lo._bf16(r.double()), bf16_by_hand(r).double())      # fp64 values that are fp32-representable
    assert torch.equal(lo._bf16(lo._bf16(r)), lo._bf16(r))                    # idempotent


@pytest.fixture(scope="module")
def runs():
    import synth_inputs as si
    g = np.random.default_rng(5)
    layers = [si.make_layer_params(CFG, 0, 5)]
    for k in ("bq", "bk", "bv", "bo", "b1", "b2", "ln1_b", "ln2_b"):
        layers[0][k] = (0.1 * g.standard_normal(layers[0][k].shape)).astype(np.float32)
    x, dy = si.make_activations(CFG, 5)
    p = lo.to_torch(layers[0])
    out = {(): lo.model_forward_backward(layers, x, dy, CFG, seed=3)}
    for s in lo.BF16_OPERAND_SITES:
        out[(s,)] = lo.model_forward_backward(layers, x, dy, CFG, seed=3, bf16_sites=(s,))
    return p, out


def _t(run, name):
    sv, it, g = run["saved"][0], run["inter"][0], run["grads"][0]
    return sv[name] if name in sv else it[name] if name in it else g[name]


def _close(a, b):
    return float((a - b).abs().max()) <= 1e-12 * max(1.0, float(b.abs().max()))


# order of computation: a tensor is upstream of a site if it is produced before the site's tensor
FORWARD_ORDER = ["u", "q", "k", "v", "P", "A", "Z1r", "x1", "v2", "f", "Z2r", "y"]
BACKWARD_ORDER = ["dZ2", "dG", "dV2r", "dx1", "dZ1", "dA", "dq", "dk", "dv", "dUr"]
SITE_TENSORS = {"u": ["u"], "qkv": ["q", "k", "v"], "A": ["A"], "v2": ["v2"], "f": ["f"], "pre": ["pre"], "dZ2": ["dZ2"], "dG": ["dG"],
                "dZ1": ["dZ1"], "dA": ["dA"], "dqkv": ["dq", "dk", "dv"]}


@pytest.mark.parametrize("site", list(SITE_TENSORS))
def test_site_rounds_its_tensor_and_nothing_upstream(runs, site):
    p, out = runs
    base, one = out[()], out[(site,)]
    order = FORWARD_ORDER + BACKWARD_ORDER
    names = SITE_TENSORS[site]
    if site == "pre":       # the stored pre-activation is rounded behind the GeLU that reads it: the whole forward is unchanged
        first = len(FORWARD_ORDER)
    else:
        first = min(order.index(n) for n in names)
    for n in order[:first]:
        assert torch.equal(_t(one, n), _t(base, n)), f"site {site}: upstream tensor {n} moved"
    for n in names:
        if site == "qkv" and n != "q":
            continue        # k and v come behind q in the order list but are not downstream of it
        assert torch.equal(_t(one, n), lo._bf16(_t(base, n))), f"site {site}: tensor {n} is not the rounded one"
    if site == "qkv":
        for n in ("k", "v"):
            assert torch.equal(_t(one, n), lo._bf16(_t(base, n)))
    changed = [n for n in order[first:] if n not in names and not torch.equal(_t(one, n), _t(base, n))]
    assert changed, f"site {site}: nothing downstream changed"


def _heads(t):
    b, s, nh = CFG["batch"], CFG["seq"], CFG["n_heads"]
    return t.reshape(b, s, nh, -1).permute(0, 2, 1, 3)


def _unheads(t):
    b, s = CFG["batch"], CFG["seq"]
    return t.permute(0, 2, 1, 3).reshape(b * s, -1)


def _softmax_causal(q, k):
    d = CFG["hidden"] // CFG["n_heads"]
    S = _heads(q) @ _heads(k).transpose(2, 3) / math.sqrt(d)
    i = torch.arange(CFG["seq"])
    return torch.softmax(S.masked_fill(i[None, :] > i[:, None], float("-inf")), dim=3)


def test_consumers_of_each_site_see_the_rounded_tensor(runs):
    p, out = runs
    base = out[()]
    bs, bi = base["saved"][0], base["inter"][0]
    r = lo._bf16
    d = CFG["hidden"] // CFG["n_heads"]
    one = lambda s: (out[(s,)]["saved"][0], out[(s,)]["inter"][0], out[(s,)]["grads"][0])
    # u: QKV reads the rounded LayerNorm output; so does the weight gradient
    sv, it, g = one("u")
    assert _close(sv["q"], r(bs["u"]) @ p["wq"] + p["bq"]) and _close(g["wk"], r(bs["u"]).t() @ it["dk"])
    # qkv: the scores and the value product read rounded q, k, v
    sv, it, g = one("qkv")
    P = _softmax_causal(r(bs["q"]), r(bs["k"]))
    assert _close(sv["A"], _unheads(P @ _heads(r(bs["v"]))))
    # P: A = round(P) V, dV = round(P)^T dA; the softmax gradient keeps the unrounded P
    sv, it, g = one("P")
    assert torch.equal(sv["P"], bs["P"])
    assert _close(sv["A"], _unheads(r(bs["P"]) @ _heads(bs["v"])))
    assert _close(it["dv"], _unheads(r(sv["P"]).transpose(2, 3) @ _heads(it["dA"])))
    # A: projection and its weight gradient
    sv, it, g = one("A")
    assert _close(sv["Z1r"], r(bs["A"]) @ p["wo"]) and _close(g["wo"], r(bs["A"]).t() @ it["dZ1"])
    # v2: FC1 and its weight gradient
    sv, it, g = one("v2")
    assert _close(sv["pre"], r(bs["v2"]) @ p["w1"] + p["b1"]) and _close(g["w1"], r(bs["v2"]).t() @ it["dG"])
    # pre: only the GeLU derivative in backward reads the stored (rounded) pre-activation
    sv, it, g = one("pre")
    assert torch.equal(sv["f"], bs["f"]) and torch.equal(out[("pre",)]["y"], base["y"])
    assert _close(it["dG"], (bi["dZ2"] @ p["w2"].t()) * lo.gelu_grad(r(bs["pre"])))
    # f: FC2 and its weight gradient
    sv, it, g = one("f")
    assert _close(sv["Z2r"], r(bs["f"]) @ p["w2"]) and _close(g["w2"], r(bs["f"]).t() @ it["dZ2"])
    # dZ2: FC2's input and weight gradients, and the bias gradient, read the rounded tensor
    sv, it, g = one("dZ2")
    dz = r(bi["dZ2"])
    assert _close(g["b2"], dz.sum(0)) and _close(g["w2"], bs["f"].t() @ dz) and _close(it["dG"], (dz @ p["w2"].t()) * lo.gelu_grad(bs["pre"]))
    # dG
    sv, it, g = one("dG")
    dg = r(bi["dG"])
    assert _close(it["dV2r"], dg @ p["w1"].t()) and _close(g["w1"], bs["v2"].t() @ dg) and _close(g["b1"], dg.sum(0))
    # dZ1
    sv, it, g = one("dZ1")
    dz = r(bi["dZ1"])
    assert _close(it["dA"], dz @ p["wo"].t()) and _close(g["wo"], bs["A"].t() @ dz) and _close(g["bo"], dz.sum(0))
    # dA: both dV = P^T dA and dP = dA V^T read the rounded tensor
    sv, it, g = one("dA")
    da = _heads(r(bi["dA"]))
    assert _close(it["dv"], _unheads(bs["P"].transpose(2, 3) @ da))
    dP = da @ _heads(bs["v"]).transpose(2, 3)
    dS = bs["P"] * (dP - (dP * bs["P"]).sum(3, keepdim=True))
    assert _close(it["dq"], _unheads(dS @ _heads(bs["k"])) / math.sqrt(d))
    # dS: dQ = round(dS) K / sqrt(d), dK = round(dS)^T Q / sqrt(d)
    sv, it, g = one("dS")
    dP = _heads(bi["dA"]) @ _heads(bs["v"]).transpose(2, 3)
    dS = r(bs["P"] * (dP - (dP * bs["P"]).sum(3, keepdim=True)))
    assert _close(it["dq"], _unheads(dS @ _heads(bs["k"])) / math.sqrt(d))
    assert _close(it["dk"], _unheads(dS.transpose(2, 3) @ _heads(bs["q"])) / math.sqrt(d))
    assert torch.equal(it["dv"], bi["dv"])
    # dqkv: QKV's input and weight gradients
    sv, it, g = one("dqkv")
    dq, dk, dv = r(bi["dq"]), r(bi["dk"]), r(bi["dv"])
    assert _close(it["dUr"], dq @ p["wq"].t() + dk @ p["wk"].t() + dv @ p["wv"].t())
    assert _close(g["wv"], bs["u"].t() @ dv) and _close(g["bq"], dq.sum(0))


def test_all_sites_together_is_each_site_applied(runs):
    """With every site on, each site's tensor is on the bf16 grid (spot check that the option composes)."""
    import synth_inputs as si
    layers = [si.make_layer_params(CFG, 0, 5)]
    x, dy = si.make_activations(CFG, 5)
    run = lo.model_forward_backward(layers, x, dy, CFG, seed=3, bf16_sites=lo.BF16_OPERAND_SITES)
    for site, names in SITE_TENSORS.items():
        for n in names:
            t = _t(run, n)
            assert torch.equal(lo._bf16(t), t), (site, n)


def test_site_list_is_what_the_library_stores_as_bf16():
    """The floor models the library's storage choices: every workspace tensor the C ABI plans with 2 bytes per element is a
    site, every fp32 one is not; P and dS are the two MFMA operands that never leave registers."""
    from paper_2305_16121_amd import binding as B
    import synth_inputs as si
    cfg = si.CONFIGS["C1"]
    H = B.Handle(B.make_cfg(cfg))
    M, h, t = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["tp"]
    hp, fp = h // t, 4 * h // t
    elems = dict(u=M * h, qkv=3 * M * hp, attn=M * hp, v2=M * h, pre=M * fp, f=M * fp, dz2=M * h, dg=M * fp, dz1=M * h, da=M * hp, dqkv=3 * M * hp,
                 z1=M * h, x1=M * h, z2=M * h, dv2=M * h, dx1=M * h, du=M * h)
    site_of = dict(u="u", qkv="qkv", attn="A", v2="v2", pre="pre", f="f", dz2="dZ2", dg="dG", dz1="dZ1", da="dA", dqkv="dqkv")
    stored_bf16 = set()
    for name, n in elems.items():
        _, nbytes = H.tensor_span(name, 0)
        assert nbytes in (2 * n, 4 * n), name
        if nbytes == 2 * n:
            stored_bf16.add(site_of[name])
        else:
            assert name not in site_of, f"{name} is fp32 in the library but a rounding site of the floor"
    assert stored_bf16 | {"P", "dS"} == set(lo.BF16_OPERAND_SITES)
