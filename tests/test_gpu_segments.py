"""Lock-step emulation of all t ranks of a partition on the one GPU, through the segment-level calls of the C ABI: every
rank runs a computation sequence up to its reduction point, the partial sums the GPU itself produced are added over the
ranks (the AllReduce y = sum_i x_i of Sec. IV-B; the addition is the harness's, as the network's would be) and the sum
is handed to every rank's next sequence -- forward and backward (Eq. (1): the gradient passes through the reduction).
No oracle value enters the GPU computation; the results are then compared with the UNSHARDED oracle."""
import pytest
import torch

import synth_inputs as si
from tests import layer_harness as LH

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def lock_step(cfg, layers, x, dy, flags=0):
    from paper_2305_16121_amd import binding as B
    t, L = cfg["tp"], cfg["n_layers"]
    M, h = x.shape
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    R = []
    for r in range(t):
        H = B.Handle(B.make_cfg(cfg, rank=r, flags=flags))
        W = [B.pack_rank_params(si.shard_layer_params(p, cfg, r)) for p in layers]
        R.append(dict(H=H, W=W, G=[B.zero_grads_like(w) for w in W],
                      ws=torch.full((H.workspace_bytes,), 0xFF, dtype=torch.uint8, device="cuda"),
                      y=torch.full((M, h), float("nan"), device="cuda"), dx=torch.full((M, h), float("nan"), device="cuda"),
                      part=torch.full((M, h), float("nan"), device="cuda")))

    def reduce_parts():     # fixed order of addition: rank 0 first
        total = R[0]["part"].clone()
        for q in R[1:]:
            total += q["part"]
        return total

    for l in range(L):
        for q in R:
            q["H"].forward_segment(l, 0, q["W"], xd, q["y"], q["ws"], partial_out=q["part"])
        z1 = reduce_parts()
        for q in R:
            q["H"].forward_segment(l, 1, q["W"], xd, q["y"], q["ws"], partial_out=q["part"], reduced_in=z1)
        z2 = reduce_parts()
        for q in R:
            q["H"].forward_segment(l, 2, q["W"], xd, q["y"], q["ws"], reduced_in=z2)
    for q in R:
        q["H"].backward_segment(L - 1, 2, q["W"], xd, dyd, q["dx"], q["G"], q["ws"])
    for l in reversed(range(L)):
        for q in R:
            q["H"].backward_segment(l, 1, q["W"], xd, dyd, q["dx"], q["G"], q["ws"], partial_out=q["part"])
        dv2 = reduce_parts()
        for q in R:
            q["H"].backward_segment(l, 0, q["W"], xd, dyd, q["dx"], q["G"], q["ws"], partial_out=q["part"], reduced_in=dv2)
        du = reduce_parts()
        for q in R:
            q["H"].backward_segment(l, 3, q["W"], xd, dyd, q["dx"], q["G"], q["ws"], reduced_in=du)
    torch.cuda.synchronize()
    return R


@pytest.mark.timeout(900)
@pytest.mark.parametrize("name", ["C1", "C2"])
def test_lock_step_ranks_reproduce_the_unsharded_layer(name):
    from oracle import layer_oracle as lo
    cfg = si.CONFIGS[name]
    layers, x, dy = LH.make_inputs(cfg)
    R = lock_step(cfg, layers, x, dy)
    # every rank holds the same residual stream: same kernels on the same reduced tensors
    for q in R[1:]:
        assert torch.equal(q["y"], R[0]["y"]) and torch.equal(q["dx"], R[0]["dx"])
    ora = lo.model_forward_backward(layers, x, dy, cfg)
    floors = [lo.model_forward_backward(layers, x, dy, cfg, dtype=dt, bf16_sites=lo.BF16_OPERAND_SITES) for dt in (torch.float64, torch.float32)]
    for r, q in enumerate(R):
        print(f"\n== {name} rank {r} of the lock-step run vs the unsharded oracle", flush=True)
        ora_r = dict(y=ora["y"], dx=ora["dx"], grads=[LH.slice_unsharded_grads(g, cfg, r) for g in ora["grads"]])
        fl_r = [dict(y=f["y"], dx=f["dx"], grads=[LH.slice_unsharded_grads(g, cfg, r) for g in f["grads"]]) for f in floors]
        gpu = dict(y=q["y"], dx=q["dx"], grads=q["G"])
        assert LH.compare_run(f"{name} rank {r}, lock-step ranks on the GPU's own partials vs unsharded", gpu, ora_r, fl_r, cfg["n_layers"])


@pytest.mark.parametrize("name,flags", [("C1", 0), ("C2", 0), ("C2", 4)])
def test_segments_back_to_back_are_the_whole_pass(name, flags):
    """With no partial / reduced tensors handed over, the segments of one rank in order give what oases_forward /
    oases_backward give without peer sums: y, dx and the weight-matrix gradients bit for bit, the bias and LayerNorm-parameter
    gradients up to the order of their fp32 column sums (also in recomputation mode, flags = 4)."""
    cfg = si.CONFIGS[name]
    layers, x, dy = LH.make_inputs(cfg)
    from paper_2305_16121_amd import binding as B
    whole = LH.gpu_rank_run(cfg, 1, layers, x, dy, flags=flags)
    M, h = x.shape
    L = cfg["n_layers"]
    H = B.Handle(B.make_cfg(cfg, rank=1, flags=flags))
    W = [B.pack_rank_params(si.shard_layer_params(p, cfg, 1)) for p in layers]
    G = [B.zero_grads_like(w) for w in W]
    ws = torch.full((H.workspace_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    y, dx = torch.full((M, h), float("nan"), device="cuda"), torch.full((M, h), float("nan"), device="cuda")
    for l in range(L):
        for seg in (0, 1, 2):
            H.forward_segment(l, seg, W, xd, y, ws)
    H.backward_segment(L - 1, 2, W, xd, dyd, dx, G, ws)
    for l in reversed(range(L)):
        for seg in (1, 0, 3):
            H.backward_segment(l, seg, W, xd, dyd, dx, G, ws)
    torch.cuda.synchronize()
    from tests.util import rel_err
    assert torch.equal(y, whole["y"]) and torch.equal(dx, whole["dx"])
    for l in range(L):
        for k in ("wqkv", "wo", "w1", "w2"):
            assert torch.equal(G[l][k], whole["grads"][l][k]), (l, k)
        # column sums: a segment adds up its own partial rows at once, the whole pass adds those of all sub-batches in one
        # launch at its end -- the same terms in another fp32 order
        for k in ("ln1_g", "ln1_b", "bqkv", "bo", "ln2_g", "ln2_b", "b1", "b2"):
            assert rel_err(G[l][k], whole["grads"][l][k]) < 1e-5, (l, k)


def test_segment_argument_errors():
    from paper_2305_16121_amd import binding as B
    cfg = si.CONFIGS["C1"]
    layers, x, dy = LH.make_inputs(cfg)
    H = B.Handle(B.make_cfg(cfg))
    W = [B.pack_rank_params(si.shard_layer_params(layers[0], cfg, 0))]
    G = [B.zero_grads_like(W[0])]
    M, h = x.shape
    xd = torch.from_numpy(x).cuda()
    y, buf = torch.empty_like(xd), torch.empty_like(xd)
    ws = torch.empty(H.workspace_bytes, dtype=torch.uint8, device="cuda")
    for args, code in [((1, 0), B.EINVAL), ((0, 3), B.EINVAL), ((0, -1), B.EINVAL)]:
        with pytest.raises(B.OasesError) as e:
            H.forward_segment(*args, W, xd, y, ws)
        assert e.value.code == code
    with pytest.raises(B.OasesError) as e:       # segment 2 ends in no reduction point
        H.forward_segment(0, 2, W, xd, y, ws, partial_out=buf)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.OasesError) as e:       # segment 0 starts from none
        H.forward_segment(0, 0, W, xd, y, ws, reduced_in=buf)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.OasesError) as e:
        H.backward_segment(0, 4, W, xd, xd, y, G, ws)
    assert e.value.code == B.EINVAL
    with pytest.raises(B.OasesError) as e:
        H.backward_segment(0, 2, W, xd, xd, y, G, ws, partial_out=buf)
    assert e.value.code == B.EINVAL
    torch.cuda.synchronize()
