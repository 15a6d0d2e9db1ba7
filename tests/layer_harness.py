"""Runs the HIP path and the oracle on the same seeded layer inputs (test infrastructure)."""
import numpy as np
import torch

import synth_inputs as si

FWD_TOL, GRAD_TOL = 1e-2, 3e-2     # max|err| / rms(ref): forward activations, weight and input gradients

GPU_PARAMS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")


def make_inputs(cfg, seed=0):
    layers = [si.make_layer_params(cfg, l, seed) for l in range(cfg["n_layers"])]
    x, dy = si.make_activations(cfg, seed)
    return layers, x, dy


def gpu_rank_run(cfg, rank, layers, x, dy, *, peers=None, n_sub=None, flags=0, seed=0, two_streams=True, keep=False):
    """One rank's forward+backward on the GPU through the C ABI.  `layers` are UNSHARDED numpy parameter dicts;
    `peers` is a list (per layer) of dicts of numpy [M,h] peer sums or None."""
    from paper_2305_16121_amd import binding as B
    M, h = x.shape
    H = B.Handle(B.make_cfg(cfg, rank=rank, seed=seed, flags=flags, n_sub=n_sub))
    W = [B.pack_rank_params(si.shard_layer_params(p, cfg, rank)) for p in layers]
    G = [B.zero_grads_like(w) for w in W]
    ws = torch.full((H.workspace_bytes,), 0xFF, dtype=torch.uint8, device="cuda")   # NaN-poisoned
    xd = torch.from_numpy(x).cuda()
    dyd = torch.from_numpy(dy).cuda()
    yd = torch.full((M, h), float("nan"), dtype=torch.float32, device="cuda")
    dxd = torch.full((M, h), float("nan"), dtype=torch.float32, device="cuda")
    P = None
    if peers is not None:
        P = [{k: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).cuda() for k, v in d.items()} for d in peers]
    s1 = torch.cuda.Stream()
    s2 = torch.cuda.Stream() if two_streams else s1
    torch.cuda.synchronize()
    H.forward(W, xd, yd, ws, peers=P, s_compute=s1, s_comm=s2)
    H.backward(W, xd, dyd, dxd, G, ws, peers=P, s_compute=s1, s_comm=s2)
    s1.synchronize()
    s2.synchronize()
    torch.cuda.synchronize()
    out = dict(y=yd, dx=dxd, grads=G)
    if keep:
        out.update(handle=H, ws=ws, weights=W)
    return out


def ws_tensor(run, name, layer, dtype, shape):
    off, nb = run["handle"].tensor_span(name, layer)
    return run["ws"][off:off + nb].view(dtype).reshape(shape)


def oracle_rank_grads_to_gpu_layout(g):
    """Oracle gradient dict (wq,wk,wv,...) -> the packed names of the library (wqkv, bqkv)."""
    out = {k: g[k] for k in ("ln1_g", "ln1_b", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")}
    out["wqkv"] = torch.cat([g["wq"], g["wk"], g["wv"]], dim=1)
    out["bqkv"] = torch.cat([g["bq"], g["bk"], g["bv"]])
    return out


def oracle_rank_only(cfg, rank, layers, x, dy, seed=0, dtype=torch.float64, bf16_sites=()):
    """The rank's computation with no peers = the layer definition on the rank's weight slices."""
    from oracle import layer_oracle as lo
    shards = [si.shard_layer_params(p, cfg, rank) for p in layers]
    return lo.model_forward_backward(shards, x, dy, cfg, seed=seed, dtype=dtype, bf16_sites=bf16_sites)


def oracle_unsharded_with_peer_sums(cfg, rank, layers, x, dy, seed=0, dtype=torch.float64):
    """Unsharded oracle run + what the other t-1 ranks would contribute at each reduction point of `rank`
    (views of the unsharded intermediates: full sum minus this rank's partial)."""
    from oracle import layer_oracle as lo
    out = lo.model_forward_backward(layers, x, dy, cfg, seed=seed, dtype=dtype)
    h, t = cfg["hidden"], cfg["tp"]
    hp, fp = h // t, 4 * h // t
    a, f = slice(rank * hp, (rank + 1) * hp), slice(rank * fp, (rank + 1) * fp)
    peers = []
    for l, p in enumerate(layers):
        w = lo.to_torch(p, dtype)
        sv, it = out["saved"][l], out["inter"][l]
        dUr = it["dq"][:, a] @ w["wq"][:, a].t() + it["dk"][:, a] @ w["wk"][:, a].t() + it["dv"][:, a] @ w["wv"][:, a].t()
        peers.append(dict(fwd_attn=(sv["Z1"] - sv["A"][:, a] @ w["wo"][a, :]).numpy(),
                          fwd_ffn=(sv["Z2"] - sv["f"][:, f] @ w["w2"][f, :]).numpy(),
                          bwd_ffn=(it["dV2"] - it["dG"][:, f] @ w["w1"][:, f].t()).numpy(),
                          bwd_attn=(it["dU"] - dUr).numpy()))
    return out, peers


def slice_unsharded_grads(g, cfg, rank):
    h, t = cfg["hidden"], cfg["tp"]
    hp, fp = h // t, 4 * h // t
    a, f = slice(rank * hp, (rank + 1) * hp), slice(rank * fp, (rank + 1) * fp)
    s = {k: g[k] for k in ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "bo", "b2")}
    for k in ("wq", "wk", "wv"):
        s[k] = g[k][:, a]
    for k in ("bq", "bk", "bv"):
        s[k] = g[k][a]
    s["wo"], s["w1"], s["b1"], s["w2"] = g["wo"][a, :], g["w1"][:, f], g["b1"][f], g["w2"][f, :]
    return s
