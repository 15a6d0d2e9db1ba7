"""Host-side checks that need no GPU: the library loads and exports every symbol the header declares,
configuration validation, workspace plan, and the operator order of the schedule against a hand
trace of the paper's Algorithm 1."""
import ctypes as C
import os
import re
import subprocess
import sys

import pytest

import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    lib = os.path.join(ROOT, "paper_2305_16121_amd", "liboases.so")
    if not os.path.exists(lib):
        subprocess.check_call([sys.executable, os.path.join(ROOT, "paper_2305_16121_amd", "csrc", "build.py")])
    from paper_2305_16121_amd import binding
    return binding


def test_every_declared_symbol_is_exported(B):
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(oases_[a-z0-9_]+)\s*\(", text)))
    assert len(names) >= 30 and "oases_plan_solve" in names and "oases_op_rope" in names
    for n in names:
        assert hasattr(B.lib, n), n


def _create(B, **over):
    cfg = dict(si.CONFIGS["C1"])
    rank = over.pop("rank", 0)
    cfg.update(over)
    c = B.make_cfg(cfg, rank=rank)
    h = C.c_void_p()
    rc = B.lib.oases_create(C.byref(c), C.byref(h))
    if rc == 0:
        B.lib.oases_destroy(h)
    return rc


def test_create_validates(B):
    assert _create(B) == 0
    assert _create(B, n_heads=7) == B.EINVAL                 # h % nh
    assert _create(B, tp=3) == B.EINVAL                      # nh % t
    assert _create(B, hidden=256, n_heads=8) == B.EINVAL     # head dim 32
    assert _create(B, rank=2) == B.EINVAL                    # r >= t
    assert _create(B, dropout_p=1.0) == B.EINVAL
    assert _create(B, dropout_p=-0.1) == B.EINVAL
    assert _create(B, n_sub=3) == B.EINVAL                   # tokens % n
    assert _create(B, n_sub=8, causal=0) == B.EINVAL         # sequence chunks need causal attention
    assert _create(B, n_sub=8, causal=1) == 0
    assert _create(B, n_sub=0) == B.EINVAL
    assert b"n_sub" in B.lib.oases_last_error()
    assert B.lib.oases_create(None, None) == B.ENULL
    for name in si.CONFIGS:
        cfg = si.CONFIGS[name]
        for r in (0, cfg["tp"] - 1):
            H = B.Handle(B.make_cfg(cfg, rank=r))
            assert H.workspace_bytes > 0
            H.close()


def test_workspace_plan(B):
    cfg = si.CONFIGS["C2"]
    H = B.Handle(B.make_cfg(cfg))
    M, h, t = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["tp"]
    spans = []
    for layer in range(cfg["n_layers"]):
        for name, nbytes in (("u", M * h * 2), ("qkv", M * 3 * h // t * 2), ("x1", M * h * 4), ("pre", M * 4 * h // t * 2),
                             ("lse", cfg["batch"] * cfg["n_heads"] // t * cfg["seq"] * 4), ("du", M * h * 4)):
            off, nb = H.tensor_span(name, layer)
            assert nb == nbytes and off % 256 == 0 and off + nb <= H.workspace_bytes
            spans.append((off, off + nb))
    spans.sort()
    assert all(a[1] <= b[0] for a, b in zip(spans, spans[1:]))      # no overlap
    with pytest.raises(B.OasesError):
        H.tensor_span("nope", 0)


# Hand trace of Algorithm 1 for one layer and two sub-batches.  Forward: the computation sequence up to a
# communication operator runs for sub-batch 0, its communication starts, the sequence is replayed for sub-batch 1;
# then the next sequence.  Backward: saved sequences are popped last-first, so sub-batch 1 leads; operators behind a
# communication operator travel with it on the communication stream; the weight-gradient GEMMs of a block run once,
# over all sub-batches' rows ("sb*"), behind the block's last reduction start.  The last operator adds up the partial rows
# of every column reduction of the pass (bias and LayerNorm-parameter gradients) in one launch.
FWD_TRACE = """\
compute LN1 sb0|compute QKV sb0|compute ATTN sb0|compute PROJ sb0|comm R1+BDR1+LN2 sb0
compute LN1 sb1|compute QKV sb1|compute ATTN sb1|compute PROJ sb1|comm R1+BDR1+LN2 sb1
compute FC1+GELU sb0|compute FC2 sb0|comm R2+BDR2 sb0
compute FC1+GELU sb1|compute FC2 sb1|comm R2+BDR2 sb1
compute join sb0|compute join sb1"""
BWD_TRACE = """\
comm BDR2.b sb1|comm BDR2.b sb0
compute FC2.dgrad+dGELU sb1|compute FC1.dgrad sb1|comm R3+LN2.b+BDR1.b sb1
compute FC2.dgrad+dGELU sb0|compute FC1.dgrad sb0|comm R3+LN2.b+BDR1.b sb0
compute FC2.wgrad sb*|compute FC1.wgrad sb*|compute b1.sum sb*
compute PROJ.dgrad sb1|compute ATTN.b sb1|compute QKV.dgrad sb1|comm R4+LN1.b sb1
compute PROJ.dgrad sb0|compute ATTN.b sb0|compute QKV.dgrad sb0|comm R4+LN1.b sb0
compute PROJ.wgrad sb*|compute QKV.wgrad sb*|compute bqkv.sum sb*
compute join sb1|compute join sb0|compute colsums sb*"""


# The same with fine-grained recomputation (Sec. IV-B): each popped sequence is first rebuilt from its stored input by the
# forward kernels (".r"), starting BEHIND the forward communication operator, so no reduction point is ever re-run.
BWD_TRACE_RECOMPUTE = """\
comm BDR2.b sb1|comm BDR2.b sb0
compute LN2.r sb1|compute FC1+GELU.r sb1|compute FC2.dgrad+dGELU sb1|compute FC1.dgrad sb1|comm R3+LN2.b+BDR1.b sb1
compute LN2.r sb0|compute FC1+GELU.r sb0|compute FC2.dgrad+dGELU sb0|compute FC1.dgrad sb0|comm R3+LN2.b+BDR1.b sb0
compute FC2.wgrad sb*|compute FC1.wgrad sb*|compute b1.sum sb*
compute LN1.r sb1|compute QKV.r sb1|compute ATTN.r sb1|compute PROJ.dgrad sb1|compute ATTN.b sb1|compute QKV.dgrad sb1|comm R4+LN1.b sb1
compute LN1.r sb0|compute QKV.r sb0|compute ATTN.r sb0|compute PROJ.dgrad sb0|compute ATTN.b sb0|compute QKV.dgrad sb0|comm R4+LN1.b sb0
compute PROJ.wgrad sb*|compute QKV.wgrad sb*|compute bqkv.sum sb*
compute join sb1|compute join sb0|compute colsums sb*"""


def _norm(trace):
    return [x.strip() for line in trace.splitlines() for x in line.split("|")]


def test_schedule_matches_hand_trace(B):
    H = B.Handle(B.make_cfg(si.CONFIGS["C1"]))
    strip = lambda s: [re.sub(r" L0", "", l) for l in s.strip().splitlines()]
    assert strip(H.schedule(False)) == _norm(FWD_TRACE)
    assert strip(H.schedule(True)) == _norm(BWD_TRACE)
    HR = B.Handle(B.make_cfg(si.CONFIGS["C1"], flags=B.FLAG_RECOMPUTE))
    assert strip(HR.schedule(False)) == _norm(FWD_TRACE)          # forward is the same
    assert strip(HR.schedule(True)) == _norm(BWD_TRACE_RECOMPUTE)


def test_recompute_mode_workspace_and_chunk_order(B):
    # stacked layers: the rebuilt activations share one region, so the workspace shrinks
    cfg = si.CONFIGS["C2"]
    a, b = B.Handle(B.make_cfg(cfg)), B.Handle(B.make_cfg(cfg, flags=B.FLAG_RECOMPUTE))
    assert b.workspace_bytes < a.workspace_bytes
    assert a.tensor_span("qkv", 0)[0] != a.tensor_span("qkv", 1)[0]
    assert b.tensor_span("qkv", 0)[0] == b.tensor_span("qkv", 1)[0]          # shared
    assert b.tensor_span("x1", 0)[0] != b.tensor_span("x1", 1)[0]            # sequence inputs stay per layer
    # sub-batches that are chunks of a sequence: K/V of every chunk are rebuilt before any chunk's attention
    c = B.Handle(B.make_cfg(si.CONFIGS["C5"], flags=B.FLAG_RECOMPUTE)).schedule(True).splitlines()
    idx = lambda op, sb: next(i for i, l in enumerate(c) if f" {op} " in l and l.endswith(f"sb{sb}"))
    assert max(idx("QKV.r", j) for j in range(4)) < min(idx("ATTN.r", j) for j in range(4))
    assert [idx("ATTN.r", j) for j in range(4)] == sorted(idx("ATTN.r", j) for j in range(4))    # earlier chunks first
    assert max(idx("ATTN.r", j) for j in range(4)) < min(idx("ATTN.b", j) for j in range(4))


@pytest.mark.parametrize("name", ["C2", "C5"])
def test_schedule_structure(B, name):
    cfg = si.CONFIGS[name]
    L, n = cfg["n_layers"], cfg["n_sub"]
    H = B.Handle(B.make_cfg(cfg))
    fwd, bwd = H.schedule(False).strip().splitlines(), H.schedule(True).strip().splitlines()
    # two reduction points per layer and pass, per sub-batch (the third, recompute one of the paper is not needed here)
    assert sum(l.startswith("comm R") for l in fwd) == 2 * L * n
    assert sum(l.startswith("comm R") for l in bwd) == 2 * L * n
    # forward: within a layer segment sub-batches go 0..n-1; backward: n-1..0
    subs = [int(l.rsplit("sb", 1)[1]) for l in fwd if " QKV " in l and " L0 " in l]
    assert subs == list(range(n))
    subs = [int(l.rsplit("sb", 1)[1]) for l in bwd if " ATTN.b " in l and " L0 " in l]
    assert subs == list(range(n - 1, -1, -1))
    # every operator of every (layer, sub-batch) appears exactly once
    for op, lines in (("QKV", fwd), ("FC2", fwd), ("QKV.dgrad", bwd), ("R4+LN1.b", bwd)):
        assert sum(f" {op} " in l for l in lines) == L * n
    for op in ("QKV.wgrad", "FC1.wgrad", "bqkv.sum"):       # merged over the sub-batches
        assert sum(f" {op} " in l for l in bwd) == L
    # LN1 is a separate operator only for the first layer (later ones ride on the layer below's R2)
    assert sum(" LN1 " in l for l in fwd) == n


def test_attention_weight_gradients_share_a_launch_where_it_pays(B):
    """PROJ.wgrad and QKV.wgrad go out as one launch when both fit whole 128 x 256 tiles, have more than 128 tiles together
    and need fewer rounds of 256 workgroups together than apart (host rule); the schedule then holds one operator for
    the two."""
    wins = B.lib.oases_op_gemm_tn_pair_wins
    assert wins(8192, 512, 4096, 4096, 1536) == 1          # C4: 64 + 192 tiles = one round instead of two
    assert wins(8192, 1024, 8192, 8192, 3072) == 0         # C5: 256 + 768 tiles, four rounds either way
    assert wins(4096, 256, 1024, 1024, 768) == 0           # C2: 32 tiles, too few for whole 128 x 256 tiles
    assert wins(8192, 512, 4096, 4096, 1408) == 0          # N not a multiple of 256
    assert wins(8200, 512, 4096, 4096, 1536) == 0          # K not a multiple of 64
    assert wins(0, 512, 4096, 4096, 1536) == 0 and wins(8192, -128, 4096, 4096, 1536) == 0
    for name, paired in (("C4", True), ("C5", False), ("C2", False)):
        cfg = si.CONFIGS[name]
        for flags in (0, B.FLAG_RECOMPUTE):
            bwd = B.Handle(B.make_cfg(cfg, flags=flags)).schedule(True).splitlines()
            count = lambda op: sum(f" {op} " in l for l in bwd)
            assert count("PROJ+QKV.wgrad") == (cfg["n_layers"] if paired else 0), name
            assert count("PROJ.wgrad") == count("QKV.wgrad") == (0 if paired else cfg["n_layers"]), name
            assert count("bqkv.sum") == cfg["n_layers"]
    bwd = B.Handle(B.make_cfg(si.LLAMA_CONFIGS["L4"])).schedule(True).splitlines()
    assert sum(" PROJ+QKV.wgrad " in l for l in bwd) == 1


def test_gemm_choice_for_the_measured_workloads(B):
    """The kernel instantiation the library picks (host query) for launches of the measured workloads: the eight-wave
    direct-to-LDS kernels wherever whole k tiles allow them, k slices only with a workspace that holds the partial planes."""
    v = B.lib.oases_op_gemm_variant
    ws = 256 << 20
    assert v(B.GEMM_TN, B.EPI_F32, 2048, 4096, 8192, ws) == 301128256          # C4: merged weight gradient of FC2
    assert v(B.GEMM_NN, B.EPI_BIAS_BF16, 4096, 1536, 4096, ws) == 301128256    # C4: QKV
    assert v(B.GEMM_NN, B.EPI_BIAS_GELU, 4096, 2048, 4096, ws) == 301128256    # C4: FC1
    assert v(B.GEMM_NT, B.EPI_F32, 4096, 4096, 2048, ws) == 301256256          # C4: FC1 input gradient
    assert v(B.GEMM_NN, B.EPI_BIAS_GELU, 1024, 4096, 8192, ws) == 302128256    # C5: few rows, long k -> two k slices
    assert v(B.GEMM_NN, B.EPI_BIAS_GELU, 1024, 4096, 8192, 0) == 1128128       # ... not without a workspace
    assert v(B.GEMM_NT, B.EPI_DGELU, 1024, 4096, 8192, ws) == 302128256
    assert v(B.GEMM_TN, B.EPI_F32, 8192, 4096, 8192, ws) == 301256256          # C5: merged weight gradient of FC1
    assert v(B.GEMM_TN, B.EPI_F32, 4096, 2752, 8192, ws) == 301256256          # L4: a ragged last tile column
    assert v(B.GEMM_NN, B.EPI_SWIGLU, 4096, 2752, 4096, ws) == 301256256       # L4: FC1 + SwiGLU
    assert v(B.GEMM_NT, B.EPI_DSWIGLU, 4096, 1376, 4096, ws) == 301128256      # L4: FC2 input gradient


# ------------------------------------------------------------------ LLaMA-style layer: schedule and configuration checks
LLAMA_FWD_TRACE = """\
compute ROPE.table sb*
compute RMS1 sb0|compute QKV sb0|compute ROPE sb0|compute ATTN sb0|compute PROJ sb0|comm R1+DR1+RMS2 sb0
compute RMS1 sb1|compute QKV sb1|compute ROPE sb1|compute ATTN sb1|compute PROJ sb1|comm R1+DR1+RMS2 sb1
compute FC1+SWIGLU sb0|compute FC2 sb0|comm R2+DR2 sb0
compute FC1+SWIGLU sb1|compute FC2 sb1|comm R2+DR2 sb1
compute join sb0|compute join sb1"""
# backward with recomputation: the rotation is redone behind QKV.r, and dQ / dK are rotated back behind the attention
# backward, before the input-gradient GEMM of QKV; no bias sums
LLAMA_BWD_TRACE_RECOMPUTE = """\
comm DR2.b sb1|comm DR2.b sb0
compute RMS2.r sb1|compute FC1+SWIGLU.r sb1|compute FC2.dgrad+dSWIGLU sb1|compute FC1.dgrad sb1|comm R3+RMS2.b+DR1.b sb1
compute RMS2.r sb0|compute FC1+SWIGLU.r sb0|compute FC2.dgrad+dSWIGLU sb0|compute FC1.dgrad sb0|comm R3+RMS2.b+DR1.b sb0
compute FC2.wgrad sb*|compute FC1.wgrad sb*
compute RMS1.r sb1|compute QKV.r sb1|compute ROPE.r sb1|compute ATTN.r sb1|compute PROJ.dgrad sb1|compute ATTN.b sb1|compute ROPE.b sb1|compute QKV.dgrad sb1|comm R4+RMS1.b sb1
compute RMS1.r sb0|compute QKV.r sb0|compute ROPE.r sb0|compute ATTN.r sb0|compute PROJ.dgrad sb0|compute ATTN.b sb0|compute ROPE.b sb0|compute QKV.dgrad sb0|comm R4+RMS1.b sb0
compute PROJ.wgrad sb*|compute QKV.wgrad sb*
compute join sb1|compute join sb0|compute colsums sb*"""


def test_llama_schedule_matches_hand_trace(B):
    strip = lambda s: [re.sub(r" L0", "", l) for l in s.strip().splitlines()]
    H = B.Handle(B.make_cfg(si.LLAMA_CONFIGS["L1"], flags=B.FLAG_RECOMPUTE))
    assert strip(H.schedule(False)) == _norm(LLAMA_FWD_TRACE)
    assert strip(H.schedule(True)) == _norm(LLAMA_BWD_TRACE_RECOMPUTE)
    stored = strip(B.Handle(B.make_cfg(si.LLAMA_CONFIGS["L1"])).schedule(True))
    assert stored == [l for l in _norm(LLAMA_BWD_TRACE_RECOMPUTE) if ".r " not in l]
    # the FC1 output kept for backward is twice as wide (gate and up), the rotary table exists
    off, nb = H.tensor_span("pre", 0)
    c = si.LLAMA_CONFIGS["L1"]
    assert nb == c["batch"] * c["seq"] * 2 * (c["ffn_hidden"] // c["tp"]) * 2
    assert H.tensor_span("rope", 0)[1] == c["seq"] * (c["hidden"] // c["n_heads"] // 2) * 8


def test_create_rejects_bad_llama_configurations(B):
    def rc(**over):
        cfg = dict(si.LLAMA_CONFIGS["L1"])
        cfg.update(over)
        c, h = B.make_cfg(cfg), C.c_void_p()
        r = B.lib.oases_create(C.byref(c), C.byref(h))
        if r == 0:
            B.lib.oases_destroy(h)
        return r
    assert rc() == 0
    assert rc(ffn_hidden=720) == B.EINVAL          # 360 columns per rank: not a multiple of 32
    assert rc(ffn_hidden=705) == B.EINVAL          # not divisible by the degree
    assert rc(rope_theta=0.5) == B.EINVAL
    c, h = B.make_cfg(si.CONFIGS["C1"]), C.c_void_p()
    c.ffn_hidden = 1024
    assert B.lib.oases_create(C.byref(c), C.byref(h)) == B.EINVAL   # the GPT layer's FFN width is 4h
    c = B.make_cfg(si.LLAMA_CONFIGS["L1"])
    c.arch = 7
    assert B.lib.oases_create(C.byref(c), C.byref(h)) == B.EINVAL


def test_bert_schedule_and_workspace(B):
    """Post-LN layer: the layer input enters QKV as a cast (no LayerNorm in front), the top of the backward pass is the
    backward of LN2 fused with the FFN branch's dropout, the sums in front of both LayerNorms are kept."""
    cfg = dict(si.CONFIGS["C2"], arch="bert", causal=0)
    H = B.Handle(B.make_cfg(cfg))
    fwd, bwd = H.schedule(False).splitlines(), H.schedule(True).splitlines()
    assert fwd[0] == "compute CAST L0 sb0" and "comm R1+BDR1+LN1 L0 sb0" in fwd and "comm R2+BDR2+LN2 L1 sb1" in fwd
    assert sum(1 for l in fwd if " CAST " in l) == cfg["n_sub"]            # only layer 0 casts: deeper layers get the bf16 copy from R2
    assert bwd[0] == "comm LN2.b+BDR2.b L1 sb1" and "comm R4+LN2.b+BDR2.b L0 sb0" in bwd
    M, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
    for name in ("s1", "s2", "ds2", "x1"):
        assert H.tensor_span(name, 1)[1] == M * h * 4
    G = B.Handle(B.make_cfg(si.CONFIGS["C2"]))
    assert G.tensor_span("s1", 0)[1] == 0 and H.workspace_bytes > G.workspace_bytes
