"""Parity of the whole path on the LLaMA-style layer (RMSNorm, rotary embedding, SwiGLU; the second model family of the
paper's Table III) against its CPU oracle, through the C ABI: rank-only runs, runs with peer sums against the
unsharded layer, sub-batch invariance (incl. sequence chunks), recomputation mode, two streams.  Tolerance policy as
in test_gpu_layer.py."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import layer_harness as LH
from tests.layer_harness import compare_run
from tests.util import rel_err

pytestmark = pytest.mark.gpu
PARAMS = ("ln1_g", "wqkv", "wo", "ln2_g", "w1", "w2")


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def make_inputs(cfg, seed=0):
    layers = [si.make_llama_layer_params(cfg, l, seed) for l in range(cfg["n_layers"])]
    x, dy = si.make_activations(cfg, seed)
    return layers, x, dy


def gpu_run(cfg, rank, layers, x, dy, *, peers=None, n_sub=None, flags=0, seed=0, two_streams=True):
    from paper_2305_16121_amd import binding as B
    M, h = x.shape
    H = B.Handle(B.make_cfg(cfg, rank=rank, seed=seed, flags=flags, n_sub=n_sub))
    W = [B.pack_llama_rank_params(si.shard_llama_layer_params(p, cfg, rank)) for p in layers]
    G = [B.zero_grads_like(w) for w in W]
    ws = torch.full((H.workspace_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
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
    torch.cuda.synchronize()
    H.close()
    return dict(y=yd, dx=dxd, grads=G)


def to_gpu_layout(g):
    """Oracle gradients (wq, wk, wv, wg, wu, ...) in the library's packed layout."""
    from paper_2305_16121_amd import binding as B
    out = {k: g[k] for k in ("ln1_g", "wo", "ln2_g", "w2")}
    out["wqkv"] = torch.cat([g["wq"], g["wk"], g["wv"]], dim=1)
    out["w1"] = torch.from_numpy(B.interleave_gate_up(g["wg"].numpy(), g["wu"].numpy()))
    return out


def oracle_rank_only(cfg, rank, layers, x, dy, seed=0, dtype=torch.float64, bf16_sites=()):
    from oracle import llama_oracle as ll
    shards = [si.shard_llama_layer_params(p, cfg, rank) for p in layers]
    return ll.model_forward_backward(shards, x, dy, cfg, seed=seed, dtype=dtype, bf16_sites=bf16_sites)


def compare(case, gpu, ora, floors, layers):
    return compare_run(case, gpu, ora, floors, layers, to_layout=to_gpu_layout)


RAGGED = dict(arch="llama", hidden=768, n_heads=6, seq=200, batch=3, tp=3, n_sub=3, n_layers=2, causal=1, dropout_p=0.2, ffn_hidden=2016,
              rope_theta=10000.0, w_sigma=0.02)                      # d=128, t=3, fp=672, rows off the tile grid
CHUNKS = dict(arch="llama", hidden=512, n_heads=8, seq=264, batch=1, tp=2, n_sub=3, n_layers=2, causal=1, dropout_p=0.0, ffn_hidden=1408,
              rope_theta=500000.0, w_sigma=0.02)                     # d=64, sub-batches are chunks of one sequence, other theta


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,ranks,dtype", [("L1", (0, 1), torch.float64), ("L2", (0, 3), torch.float64), ("ragged", (0, 2), torch.float64),
                                              ("chunks", (1,), torch.float64), ("L4", (0,), torch.float32)])
def test_rank_shard_matches_oracle(name, ranks, dtype):
    from oracle import llama_oracle as ll
    cfg = {"ragged": RAGGED, "chunks": CHUNKS}.get(name) or si.LLAMA_CONFIGS[name]
    layers, x, dy = make_inputs(cfg, seed=2)
    for r in ranks:
        print(f"\n== {name} rank {r}: rank-only LLaMA-style layer", flush=True)
        gpu = gpu_run(cfg, r, layers, x, dy, seed=7)
        ora = oracle_rank_only(cfg, r, layers, x, dy, seed=7, dtype=dtype)
        fl = [oracle_rank_only(cfg, r, layers, x, dy, seed=7, dtype=dt, bf16_sites=ll.LLAMA_BF16_OPERAND_SITES) for dt in (torch.float64, torch.float32)]
        assert compare(f"LLaMA-style {name} rank {r}, rank-only", gpu, ora, fl, cfg["n_layers"]), f"{name} rank {r}"
        del gpu, ora, fl
        torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["L1", "L2"])
def test_with_peer_sums_every_rank_gives_the_unsharded_result(name):
    from oracle import llama_oracle as ll
    cfg = si.LLAMA_CONFIGS[name]
    layers, x, dy = make_inputs(cfg)
    full = ll.model_forward_backward(layers, x, dy, cfg)
    fl_fulls = [ll.model_forward_backward(layers, x, dy, cfg, dtype=dt, bf16_sites=ll.LLAMA_BF16_OPERAND_SITES) for dt in (torch.float64, torch.float32)]
    h, t, F = cfg["hidden"], cfg["tp"], cfg["ffn_hidden"]
    hp, fp = h // t, F // t
    for r in range(t):
        a, f = slice(r * hp, (r + 1) * hp), slice(r * fp, (r + 1) * fp)
        peers = []
        for l, p in enumerate(layers):
            w = {k: torch.from_numpy(v).double() for k, v in p.items()}
            sv, it = full["saved"][l], full["inter"][l]
            dUr = it["dq"][:, a] @ w["wq"][:, a].t() + it["dk"][:, a] @ w["wk"][:, a].t() + it["dv"][:, a] @ w["wv"][:, a].t()
            dV2r = it["dgate"][:, f] @ w["wg"][:, f].t() + it["dup"][:, f] @ w["wu"][:, f].t()
            peers.append(dict(fwd_attn=(sv["Z1"] - sv["A"][:, a] @ w["wo"][a, :]).numpy(), fwd_ffn=(sv["Z2"] - sv["f"][:, f] @ w["w2"][f, :]).numpy(),
                              bwd_ffn=(it["dV2"] - dV2r).numpy(), bwd_attn=(it["dU"] - dUr).numpy()))
        print(f"\n== {name} rank {r} with peer sums vs the unsharded oracle", flush=True)
        gpu = gpu_run(cfg, r, layers, x, dy, peers=peers)

        def sl(g):
            s = {k: g[k] for k in ("ln1_g", "ln2_g")}
            for k in ("wq", "wk", "wv"):
                s[k] = g[k][:, a]
            s["wo"], s["w2"], s["wg"], s["wu"] = g["wo"][a, :], g["w2"][f, :], g["wg"][:, f], g["wu"][:, f]
            return s
        ora_r = dict(y=full["y"], dx=full["dx"], grads=[sl(g) for g in full["grads"]])
        fl_r = [dict(y=f["y"], dx=f["dx"], grads=[sl(g) for g in f["grads"]]) for f in fl_fulls]
        assert compare(f"LLaMA-style {name} rank {r}, peer sums vs unsharded", gpu, ora_r, fl_r, cfg["n_layers"]), f"{name} rank {r}"


@pytest.mark.parametrize("name,subs", [("L1", (1, 2, 4, 8)), ("L2", (1, 2, 8))])
def test_sub_batch_count_does_not_change_results(name, subs):
    """Same rows, other split (n_sub > batch: chunks of a sequence): equal up to the summation order of GEMMs whose k
    range the launcher may split differently."""
    cfg = si.LLAMA_CONFIGS[name]
    layers, x, dy = make_inputs(cfg)
    base = gpu_run(cfg, 0, layers, x, dy, n_sub=subs[0])
    for n in subs[1:]:
        run = gpu_run(cfg, 0, layers, x, dy, n_sub=n)
        assert rel_err(run["y"], base["y"]) < 5e-3 and rel_err(run["dx"], base["dx"]) < 1e-2, n
        for l in range(cfg["n_layers"]):
            for k in PARAMS:
                assert rel_err(run["grads"][l][k], base["grads"][l][k]) < LH.GRAD_TOL, (n, l, k)


@pytest.mark.parametrize("name,n_sub", [("L1", None), ("L2", None), ("L2", 8)])
def test_recompute_mode_and_one_stream_are_bit_identical(name, n_sub):
    from paper_2305_16121_amd import binding as B
    cfg = si.LLAMA_CONFIGS[name]
    layers, x, dy = make_inputs(cfg)
    base = gpu_run(cfg, 1, layers, x, dy, n_sub=n_sub)
    for flags, two in ((B.FLAG_RECOMPUTE, True), (0, False), (B.FLAG_RECOMPUTE | B.FLAG_SERIALISE, True)):
        run = gpu_run(cfg, 1, layers, x, dy, n_sub=n_sub, flags=flags, two_streams=two)
        assert torch.equal(run["y"], base["y"]) and torch.equal(run["dx"], base["dx"]), flags
        for l in range(cfg["n_layers"]):
            for k in PARAMS:
                assert torch.equal(run["grads"][l][k], base["grads"][l][k]), (flags, l, k)
