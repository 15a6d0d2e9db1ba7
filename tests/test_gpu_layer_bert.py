"""Parity of the whole path on the post-LayerNorm (BERT-style) layer against its CPU oracle, through the C ABI:
rank-only runs, runs with peer sums against the unsharded layer, sub-batch invariance, recomputation mode, one stream.
Tolerance policy as in test_gpu_layer.py."""
import pytest
import torch

import synth_inputs as si
from tests import layer_harness as LH
from tests.layer_harness import compare_run
from tests.util import rel_err

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def bert(name, **over):
    c = dict(si.CONFIGS[name], arch="bert", causal=0)
    c.update(over)
    return c


CONFIGS = {
    "B1": bert("C1"),
    "B2": bert("C2", batch=4),                                                        # BERT-large width, two layers, p = 0.1
    "B3": bert("C3", batch=4),                                                        # BERT-1.3B width
    "ragged": dict(arch="bert", hidden=768, n_heads=12, seq=72, batch=6, tp=3, n_sub=3, n_layers=3, causal=0, dropout_p=0.2, w_sigma=0.02),
    "chunks": dict(arch="bert", hidden=512, n_heads=4, seq=264, batch=1, tp=2, n_sub=3, n_layers=2, causal=1, dropout_p=0.1, w_sigma=0.02),
}


def oracle_rank_only(cfg, rank, layers, x, dy, seed=0, dtype=torch.float64, bf16_sites=()):
    from oracle import bert_oracle as bo
    shards = [si.shard_layer_params(p, cfg, rank) for p in layers]
    return bo.model_forward_backward(shards, x, dy, cfg, seed=seed, dtype=dtype, bf16_sites=bf16_sites)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name,ranks,dtype", [("B1", (0, 1), torch.float64), ("B2", (0, 3), torch.float64), ("ragged", (0, 2), torch.float64),
                                              ("chunks", (1,), torch.float64), ("B3", (0,), torch.float32)])
def test_rank_shard_matches_oracle(name, ranks, dtype):
    from oracle import bert_oracle as bo
    cfg = CONFIGS[name]
    layers, x, dy = LH.make_inputs(cfg, seed=4)
    for r in ranks:
        print(f"\n== {name} rank {r}: rank-only post-LN layer", flush=True)
        gpu = LH.gpu_rank_run(cfg, r, layers, x, dy, seed=9)
        ora = oracle_rank_only(cfg, r, layers, x, dy, seed=9, dtype=dtype)
        fl = [oracle_rank_only(cfg, r, layers, x, dy, seed=9, dtype=dt, bf16_sites=bo.BERT_BF16_OPERAND_SITES) for dt in (torch.float64, torch.float32)]
        assert compare_run(f"post-LN {name} rank {r}, rank-only", gpu, ora, fl, cfg["n_layers"]), f"{name} rank {r}"
        del gpu, ora, fl
        torch.cuda.empty_cache()


@pytest.mark.parametrize("name", ["B1", "B2"])
def test_with_peer_sums_every_rank_gives_the_unsharded_result(name):
    from oracle import bert_oracle as bo
    cfg = CONFIGS[name]
    layers, x, dy = LH.make_inputs(cfg)
    full = bo.model_forward_backward(layers, x, dy, cfg)
    fl_fulls = [bo.model_forward_backward(layers, x, dy, cfg, dtype=dt, bf16_sites=bo.BERT_BF16_OPERAND_SITES) for dt in (torch.float64, torch.float32)]
    h, t = cfg["hidden"], cfg["tp"]
    hp, fp = h // t, 4 * h // t
    for r in range(t):
        a, f = slice(r * hp, (r + 1) * hp), slice(r * fp, (r + 1) * fp)
        peers = []
        for l, p in enumerate(layers):
            w = {k: torch.from_numpy(v).double() for k, v in p.items()}
            sv, it = full["saved"][l], full["inter"][l]
            dUr = it["dq"][:, a] @ w["wq"][:, a].t() + it["dk"][:, a] @ w["wk"][:, a].t() + it["dv"][:, a] @ w["wv"][:, a].t()
            peers.append(dict(fwd_attn=(sv["Z1"] - sv["A"][:, a] @ w["wo"][a, :]).numpy(), fwd_ffn=(sv["Z2"] - sv["f"][:, f] @ w["w2"][f, :]).numpy(),
                              bwd_ffn=(it["dV2"] - it["dG"][:, f] @ w["w1"][:, f].t()).numpy(), bwd_attn=(it["dU"] - dUr).numpy()))
        print(f"\n== {name} rank {r} with peer sums vs the unsharded oracle", flush=True)
        gpu = LH.gpu_rank_run(cfg, r, layers, x, dy, peers=peers)
        ora_r = dict(y=full["y"], dx=full["dx"], grads=[LH.slice_unsharded_grads(g, cfg, r) for g in full["grads"]])
        fl_r = [dict(y=f["y"], dx=f["dx"], grads=[LH.slice_unsharded_grads(g, cfg, r) for g in f["grads"]]) for f in fl_fulls]
        assert compare_run(f"post-LN {name} rank {r}, peer sums vs unsharded", gpu, ora_r, fl_r, cfg["n_layers"]), f"{name} rank {r}"


@pytest.mark.parametrize("name,subs", [("B1", (1, 2, 4)), ("B2", (1, 2, 4))])
def test_sub_batch_count_does_not_change_results(name, subs):
    cfg = CONFIGS[name]
    layers, x, dy = LH.make_inputs(cfg)
    base = LH.gpu_rank_run(cfg, 0, layers, x, dy, n_sub=subs[0])
    for n in subs[1:]:
        run = LH.gpu_rank_run(cfg, 0, layers, x, dy, n_sub=n)
        assert rel_err(run["y"], base["y"]) < 5e-3 and rel_err(run["dx"], base["dx"]) < 1e-2, n
        for l in range(cfg["n_layers"]):
            for k in LH.GPU_PARAMS:
                assert rel_err(run["grads"][l][k], base["grads"][l][k]) < LH.GRAD_TOL, (n, l, k)


@pytest.mark.parametrize("name", ["B1", "B2", "chunks"])
def test_recompute_mode_and_one_stream_are_bit_identical(name):
    from paper_2305_16121_amd import binding as B
    cfg = CONFIGS[name]
    layers, x, dy = LH.make_inputs(cfg)
    base = LH.gpu_rank_run(cfg, 1, layers, x, dy)
    for flags, two in ((B.FLAG_RECOMPUTE, True), (0, False), (B.FLAG_RECOMPUTE | B.FLAG_SERIALISE, True)):
        run = LH.gpu_rank_run(cfg, 1, layers, x, dy, flags=flags, two_streams=two)
        assert torch.equal(run["y"], base["y"]) and torch.equal(run["dx"], base["dx"]), flags
        for l in range(cfg["n_layers"]):
            for k in LH.GPU_PARAMS:
                assert torch.equal(run["grads"][l][k], base["grads"][l][k]), (flags, l, k)
