"""The two passes enqueue only kernels and event record / wait pairs between the two streams, so a caller may capture
them into a HIP graph (serving loops, launch-bound small layers).  A replayed graph must reproduce the eager results
bit for bit, on every replay, with eager work and synchronisations of the program in between."""
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["C1", "L1"])
def test_forward_backward_under_graph_capture(name):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_16121_amd import binding as B
    llama = name.startswith("L")
    cfg = (si.LLAMA_CONFIGS if llama else si.CONFIGS)[name]
    x, dy = si.make_activations(cfg, 0)
    if llama:
        W = [B.pack_llama_rank_params(si.shard_llama_layer_params(si.make_llama_layer_params(cfg, 0, 0), cfg, 0))]
    else:
        W = [B.pack_rank_params(si.shard_layer_params(si.make_layer_params(cfg, 0, 0), cfg, 0))]
    G = [B.zero_grads_like(W[0])]
    H = B.Handle(B.make_cfg(cfg, rank=0, seed=3))
    ws = torch.full((H.workspace_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    yd, dxd = torch.empty_like(xd), torch.empty_like(xd)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()

    def step():
        H.forward(W, xd, yd, ws, s_compute=s1, s_comm=s2)
        H.backward(W, xd, dyd, dxd, G, ws, s_compute=s1, s_comm=s2)

    def zero_grads():
        for t in G[0].values():
            t.zero_()

    # eager reference (twice: the first call creates the handle's events)
    for _ in range(2):
        zero_grads()
        torch.cuda.synchronize()
        step()
        torch.cuda.synchronize()
    ref = dict(y=yd.clone(), dx=dxd.clone(), g={k: v.clone() for k, v in G[0].items()})

    g = torch.cuda.CUDAGraph()
    zero_grads()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=s1):       # capture on the compute stream; the communication stream forks from and joins it
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        zero_grads()
        yd.fill_(float("nan"))
        dxd.fill_(float("nan"))
        junk = (xd * 2.0).sum()                # eager work of the program between replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(yd, ref["y"]) and torch.equal(dxd, ref["dx"]), rep
        for k, v in G[0].items():
            assert torch.equal(v, ref["g"][k]), (rep, k)
        assert bool(torch.isfinite(junk))
    H.close()
