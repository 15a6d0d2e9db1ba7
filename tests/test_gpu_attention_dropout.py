"""Dropout on the attention probabilities: the attention kernels against the oracle's operator with the same Philox
mask (forward, backward, row ranges inside a sequence), and the whole layer with attn_dropout_p > 0 for the three layer
families (rank-only and with peer sums against the unsharded layer: the mask is keyed by the global head index)."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from tests import layer_harness as LH
from tests.layer_harness import check_tensor, compare_run
from tests.util import rms_err, bf16_round, assert_bf16_close, dev, randn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_16121_amd import binding
    return binding


@pytest.fixture(scope="module")
def lo():
    from oracle import layer_oracle
    return layer_oracle


@pytest.mark.parametrize("batch,seq,heads,d,causal,p", [(2, 256, 2, 64, 1, 0.1), (2, 192, 2, 128, 1, 0.3), (3, 200, 1, 64, 0, 0.1),
                                                        (1, 328, 2, 128, 0, 0.5), (2, 72, 3, 64, 1, 0.1)])
def test_attention_dropout_fwd_bwd(B, lo, batch, seq, heads, d, causal, p):
    g = torch.Generator().manual_seed(21)
    M, hp = batch * seq, heads * d
    seed, layer, head0, heads_total = 0xFEEDFACE12345678, 2, 3, heads + 5
    qkv = bf16_round(randn(g, M, 3 * hp))
    dout = bf16_round(randn(g, M, hp))
    q, k, v = qkv[:, :hp], qkv[:, hp:2 * hp], qkv[:, 2 * hp:]
    drop = lo.attention_dropout_factor(seed, layer, batch, seq, heads_total, head0, heads, p)
    A, P = lo.attention_fwd(q, k, v, batch, seq, heads, d, causal, drop=drop)
    qd, dod = dev(qkv, torch.bfloat16), dev(dout, torch.bfloat16)
    out = torch.zeros(M, hp, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(batch * heads * seq, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_attention_dropout_fwd(qd.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, seq, heads, d, causal, 0, M, seed, layer, p,
                                                 head0, heads_total, None))
    scale = 256.0 / (256.0 - round(256 * p))
    assert_bf16_close(out.float(), A, 0.0, 2.0 ** -9 * scale * float(v.abs().max()), 'attention forward with dropout')
    # the log-sum-exp is that of the undropped scores
    S = (lo._heads(q, batch, seq, heads, d) @ lo._heads(k, batch, seq, heads, d).transpose(2, 3)) / math.sqrt(d)
    if causal:
        i = torch.arange(seq)
        S = S.masked_fill(i[None, :] > i[:, None], float("-inf"))
    assert float((lse.cpu().double().reshape(batch, heads, seq) - torch.logsumexp(S, dim=3)).abs().max()) < 2e-3
    dq, dk, dv = lo.attention_bwd(dout, q, k, v, P, batch, seq, heads, d, drop=drop)
    dqkv = torch.zeros(M, 3 * hp, dtype=torch.bfloat16, device="cuda")
    delta = torch.zeros_like(lse)
    B.check(B.lib.oases_op_attention_dropout_bwd(qd.data_ptr(), out.data_ptr(), dod.data_ptr(), lse.data_ptr(), delta.data_ptr(), dqkv.data_ptr(),
                                                 batch, seq, heads, d, causal, 0, M, seed, layer, p, head0, heads_total, None))
    got = dqkv.float().cpu().double()
    got = dict(dq=got[:, :hp], dk=got[:, hp:2 * hp], dv=got[:, 2 * hp:])
    for name, ref in (("dq", dq), ("dk", dk), ("dv", dv)):
        assert rms_err(got[name], ref) < 8e-3, name
    # the same mathematics with the kernel's storage roundings written out (as in the test without dropout)
    H = lambda t: lo._heads(t, batch, seq, heads, d)
    U = lambda t: lo._unheads(t, batch, seq, heads, d)
    Og = out.float().cpu().double()
    dl = (H(dout) * H(Og)).sum(dim=3, keepdim=True)
    dP = (H(dout) @ H(v).transpose(2, 3)) * drop
    dS = P * (dP - dl)
    ref_b = dict(dv=U(bf16_round(P * drop).transpose(2, 3) @ H(dout)), dq=U(bf16_round(dS) @ H(k)) / math.sqrt(d),
                 dk=U(bf16_round(dS).transpose(2, 3) @ H(q)) / math.sqrt(d))
    for name in ("dq", "dk", "dv"):
        r = ref_b[name]
        assert_bf16_close(got[name], r, 3e-3, 6e-3 * float(torch.sqrt((r ** 2).mean())), name)
    # rate 0 through the same entry points = the kernels without dropout, bit for bit
    out0, out1 = torch.zeros_like(out), torch.zeros_like(out)
    B.check(B.lib.oases_op_attention_dropout_fwd(qd.data_ptr(), out0.data_ptr(), lse.data_ptr(), batch, seq, heads, d, causal, 0, M, seed, layer, 0.0,
                                                 head0, heads_total, None))
    B.check(B.lib.oases_op_attention_fwd(qd.data_ptr(), out1.data_ptr(), lse.data_ptr(), batch, seq, heads, d, causal, 0, M, None))
    assert torch.equal(out0, out1)


def test_attention_dropout_chunks_and_errors(B):
    """Row ranges inside a sequence see the same mask as a whole-sequence call (it is a function of positions)."""
    g = torch.Generator().manual_seed(22)
    batch, seq, heads, d, nchunk = 2, 256, 2, 64, 4
    M, hp = batch * seq, heads * d
    qd = dev(bf16_round(randn(g, M, 3 * hp)), torch.bfloat16)
    dod = dev(bf16_round(randn(g, M, hp)), torch.bfloat16)
    res = []
    for split in (False, True):
        out = torch.zeros(M, hp, dtype=torch.bfloat16, device="cuda")
        lse = torch.zeros(batch * heads * seq, dtype=torch.float32, device="cuda")
        dqkv = torch.zeros(M, 3 * hp, dtype=torch.bfloat16, device="cuda")
        delta = torch.zeros_like(lse)
        rows = seq // nchunk if split else M
        starts = list(range(0, M, rows))
        for r0 in starts:
            B.check(B.lib.oases_op_attention_dropout_fwd(qd.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, seq, heads, d, 1, r0, rows, 5, 1, 0.2, 0, heads, None))
        for r0 in reversed(starts):
            B.check(B.lib.oases_op_attention_dropout_bwd(qd.data_ptr(), out.data_ptr(), dod.data_ptr(), lse.data_ptr(), delta.data_ptr(), dqkv.data_ptr(),
                                                         batch, seq, heads, d, 1, r0, rows, 5, 1, 0.2, 0, heads, None))
        torch.cuda.synchronize()
        res.append((out.clone(), lse.clone(), dqkv.clone()))
    for a, b in zip(*res):
        assert torch.equal(a, b)
    out = torch.zeros(M, hp, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(batch * heads * seq, dtype=torch.float32, device="cuda")
    bad = lambda p, h0, ht: B.lib.oases_op_attention_dropout_fwd(qd.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, seq, heads, d, 1, 0, M, 5, 1, p, h0, ht, None)
    assert bad(1.0, 0, heads) == B.EINVAL and bad(-0.1, 0, heads) == B.EINVAL and bad(0.2, 1, heads) == B.EINVAL and bad(0.2, 0, 0) == B.EINVAL
    torch.cuda.synchronize()


def _oracle(arch):
    if arch == "llama":
        from oracle import llama_oracle as m
        return m, m.LLAMA_BF16_OPERAND_SITES
    if arch == "bert":
        from oracle import bert_oracle as m
        return m, m.BERT_BF16_OPERAND_SITES
    from oracle import layer_oracle as m
    return m, m.BF16_OPERAND_SITES


@pytest.mark.parametrize("arch", ["gpt", "bert"])
def test_layer_with_attention_dropout(arch):
    """Whole layer, attn_dropout_p = 0.1 beside the hidden dropouts: rank-only for the last rank (its heads are not the
    first ones) and, with peer sums, against the unsharded layer."""
    mod, sites = _oracle(arch)
    cfg = dict(si.CONFIGS["C2"], attn_dropout_p=0.1, batch=4)
    if arch == "bert":
        cfg.update(arch="bert", causal=0)
    layers, x, dy = LH.make_inputs(cfg, seed=6)
    t, r = cfg["tp"], cfg["tp"] - 1
    heads_l = cfg["n_heads"] // t
    shards = [si.shard_layer_params(p, cfg, r) for p in layers]
    gpu = LH.gpu_rank_run(cfg, r, layers, x, dy, seed=13)
    ora = mod.model_forward_backward(shards, x, dy, cfg, seed=13, head0=r * heads_l)
    fl = [mod.model_forward_backward(shards, x, dy, cfg, seed=13, head0=r * heads_l, dtype=dt, bf16_sites=sites) for dt in (torch.float64, torch.float32)]
    assert compare_run(f"{arch} C2-like with attention dropout, rank {r}, rank-only", gpu, ora, fl, cfg["n_layers"])
    # the run is not the one without attention dropout
    cfg0 = dict(cfg, attn_dropout_p=0.0)
    gpu0 = LH.gpu_rank_run(cfg0, r, layers, x, dy, seed=13)
    assert float((gpu0["y"] - gpu["y"]).abs().max()) > 1e-2
    # sub-batch split and recomputation do not move the mask
    from paper_2305_16121_amd import binding as B
    again = LH.gpu_rank_run(cfg, r, layers, x, dy, seed=13, flags=B.FLAG_RECOMPUTE)
    assert torch.equal(again["y"], gpu["y"]) and torch.equal(again["dx"], gpu["dx"])
    chunks = LH.gpu_rank_run(dict(cfg, causal=1), r, layers, x, dy, seed=13, n_sub=2)
    chunks8 = LH.gpu_rank_run(dict(cfg, causal=1), r, layers, x, dy, seed=13, n_sub=8)      # 8 > batch: chunks of a sequence
    assert float((chunks8["y"] - chunks["y"]).abs().max()) / float(chunks["y"].abs().max()) < 5e-3
