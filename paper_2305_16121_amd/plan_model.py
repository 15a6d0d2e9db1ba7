"""Offline profiling + planning for a stack of identical layers (the offline profiling step of paper Sec. V-C): run ONE layer
of the model on this GPU under every power-of-two TMP degree with the library's per-operator timers, turn the
timings into the cost vectors of Eq. (3), model communication, AllGather and memory analytically, and let the
library's planner (include/oases_planner.h) choose a degree per layer.

    python -m paper_2305_16121_amd.plan_model --config C4 --layers 32 --capacity-gb 64

What is measured: d^0, d^1 (forward and backward, the backward under fine-grained recomputation as Sec. IV-B runs
it) of the two blocks of a layer -- [LN1, QKV, ATTN, PROJ | reduction] and [BDR1+LN2, FC1, FC2 | reduction]; the
kernel that consumes a reduction belongs to the block that follows it in the pass.  A weight-gradient GEMM that is
merged over the sub-batches is charged half to each.
What is modelled (one node of `--gpus` GPUs, all-to-all links of `--link-gbs` GB/s each way, AllReduce volume 2K(N-1)/N as in Sec. V):
  AllReduce of a sub-batch partial, K = Ms*h*4 bytes, N = degree:  ring  2K(N-1)/N / link,  mesh  2K/N / link
  AllGather on a change of degree (the activation [Ms, h] fp32):   ring  K(N-1)/N / link,   mesh  K/N / link, N = larger degree
  m_s = 16 bytes per parameter of the block / degree; m_t = the block's saved input, M_local*h*4 bytes;
  m_r = the library's workspace for one layer in recomputation mode.
The global batch is fixed: a degree-N group of the node gets global_batch * N / gpus sequences.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

FWD_BLOCK = {"LN1": 0, "QKV": 0, "ATTN": 0, "PROJ": 0, "R1+BDR1+LN2": 1, "FC1+GELU": 1, "FC2": 1, "R2+BDR2": 0}
BWD_BLOCK = {"BDR2.b": 1, "LN2.r": 1, "FC1+GELU.r": 1, "FC2.dgrad+dGELU": 1, "FC1.dgrad": 1, "FC2.wgrad": 1, "FC1.wgrad": 1, "b1.sum": 1,
             "R3+LN2.b+BDR1.b": 0, "LN1.r": 0, "QKV.r": 0, "ATTN.r": 0, "PROJ.dgrad": 0, "ATTN.b": 0, "QKV.dgrad": 0, "PROJ.wgrad": 0,
             "QKV.wgrad": 0, "PROJ+QKV.wgrad": 0, "bqkv.sum": 0, "R4+LN1.b": 1,
             "colsums": 0}   # second stage of all column reductions of the pass (last operator): charged to the attention block


def profile_degree(cfg, reps):
    """-> {"f": [[d0, d1] per block], "b": [[d0, d1] per block], "workspace": bytes} in milliseconds, for cfg["tp"]."""
    import torch
    import synth_inputs as si
    from . import binding as B
    p = si.make_layer_params(cfg, 0, 0)
    W = [B.pack_rank_params(si.shard_layer_params(p, cfg, 0))]
    G = [B.zero_grads_like(W[0])]
    x, dy = si.make_activations(cfg, 0)
    xd, dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
    yd, dxd = torch.empty_like(xd), torch.empty_like(xd)
    H = B.Handle(B.make_cfg(cfg, rank=0, seed=0, flags=B.FLAG_SERIALISE | B.FLAG_PROFILE | B.FLAG_RECOMPUTE))
    ws = torch.empty(H.workspace_bytes, dtype=torch.uint8, device="cuda")
    s1 = torch.cuda.Stream()
    out = {"f": [[0.0, 0.0], [0.0, 0.0]], "b": [[0.0, 0.0], [0.0, 0.0]], "workspace": H.workspace_bytes}
    for rep in range(reps + 1):
        H.forward(W, xd, yd, ws, s_compute=s1, s_comm=s1)
        H.backward(W, xd, dyd, dxd, G, ws, s_compute=s1, s_comm=s1)
        torch.cuda.synchronize()
        if rep == 0:
            continue
        for bwd, table, key in ((False, FWD_BLOCK, "f"), (True, BWD_BLOCK, "b")):
            for line, ms in H.profile(bwd):
                _, op, _layer, sb = line.split()[:4]
                if op == "join":
                    continue
                blk = table[op]
                if sb == "sb*":
                    out[key][blk][0] += ms / 2 / reps
                    out[key][blk][1] += ms / 2 / reps
                else:
                    out[key][blk][int(sb[2:]) % 2] += ms / reps
    H.close()
    return out


def build_problem(cfg, degrees, prof, layers, gpus, link_gbs, comm, capacity_gb, tie_layer=True):
    h, s = cfg["hidden"], cfg["seq"]
    n, p = 2 * layers, len(degrees)
    link = link_gbs * 1e9
    q = {"n_nodes": n, "n_strategies": p}
    for name in ("d0_f", "d1_f", "c0_f", "c1_f", "d0_b", "d1_b", "c0_b", "c1_b", "m_s", "m_t"):
        q[name] = [[0.0] * p for _ in range(n)]
    q["m_r"] = [0.0] * p
    K = []
    for j, t in enumerate(degrees):
        b_local = cfg["global_batch"] * t // gpus
        k_bytes = b_local * s // 2 * h * 4          # one sub-batch's partial, fp32
        K.append(k_bytes)
        c_ms = 0.0 if t == 1 else (2 * k_bytes * (t - 1) / t if comm == "ring" else 2 * k_bytes / t) / link * 1e3
        q["m_r"][j] = float(prof[t]["workspace"])
        for v in range(n):
            blk = v % 2
            q["d0_f"][v][j], q["d1_f"][v][j] = prof[t]["f"][blk]
            q["d0_b"][v][j], q["d1_b"][v][j] = prof[t]["b"][blk]
            for name in ("c0_f", "c1_f", "c0_b", "c1_b"):
                q[name][v][j] = c_ms
            q["m_s"][v][j] = 16.0 * (4 if blk == 0 else 8) * h * h / t
            q["m_t"][v][j] = float(b_local * s * h * 4)
    ag = [[0.0] * p for _ in range(p)]
    for i, ti in enumerate(degrees):
        for j, tj in enumerate(degrees):
            if i != j:
                big, kb = max(ti, tj), max(K[i], K[j])
                ag[i][j] = (kb * (big - 1) / big if comm == "ring" else kb / big) / link * 1e3 * 2     # both sub-batches
    q["t_ag_f"] = q["t_ag_b"] = [ag for _ in range(n - 1)]
    q["m"] = capacity_gb * 1e9
    if tie_layer:
        q["tie"] = [1 if v % 2 == 0 else 0 for v in range(n - 1)]
    return q


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", default="C4")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--gpus", type=int, default=8, help="GPUs of the node that the TMP groups are carved from")
    ap.add_argument("--global-batch", type=int, default=8, help="sequences per iteration over the whole node")
    ap.add_argument("--degrees", default="1,2,4,8")
    ap.add_argument("--link-gbs", type=float, default=153.0)
    ap.add_argument("--comm", choices=("ring", "mesh"), default="mesh")
    ap.add_argument("--capacity-gb", type=float, nargs="+", default=[288.0, 48.0, 35.0])
    ap.add_argument("--reps", type=int, default=5)
    a = ap.parse_args()
    import torch
    import synth_inputs as si
    from . import planner as P
    if not torch.cuda.is_available():
        sys.exit("plan_model: no GPU visible (the cost vectors are measured, there is no CPU fallback)")
    degrees = [int(t) for t in a.degrees.split(",")]
    base = dict(si.CONFIGS[a.config])
    base.update(n_layers=1, n_sub=2, global_batch=a.global_batch)
    prof = {}
    for t in degrees:
        cfg = dict(base)
        cfg.update(tp=t, batch=a.global_batch * t // a.gpus)
        if cfg["batch"] < 1 or base["n_heads"] % t:
            sys.exit(f"plan_model: degree {t} does not divide the batch / heads")
        prof[t] = profile_degree(cfg, a.reps)
        print(f"# degree {t}: batch {cfg['batch']}  fwd blocks {prof[t]['f']}  bwd blocks {prof[t]['b']} ms  workspace {prof[t]['workspace'] / 2**30:.2f} GiB",
              file=sys.stderr, flush=True)
    results = []
    for cap in a.capacity_gb:
        q = build_problem(base, degrees, prof, a.layers, a.gpus, a.link_gbs, a.comm, cap)
        t0 = time.perf_counter()
        s, cost, mem = P.plan_solve(q)
        solve_ms = (time.perf_counter() - t0) * 1e3
        row = {"capacity_gb": cap, "solve_ms": round(solve_ms, 2)}
        if s is None:
            row["strategy"] = None
        else:
            per_layer = [degrees[s[2 * l]] for l in range(a.layers)]
            groups, last = [], None
            for t in per_layer:
                if t == last:
                    groups[-1][1] += 1
                else:
                    groups.append([t, 1]); last = t
            parts = P.plan_cost(q, s)
            row.update(strategy="+".join(f"[{t}]x{c}" for t, c in groups), cost_ms=round(cost, 3), reshard_ms=round(parts["edges"], 3),
                       memory_gb=round(mem / 1e9, 2))
            for j, t in enumerate(degrees):
                uni = [j] * (2 * a.layers)
                pc = P.plan_cost(q, uni)
                row[f"uniform_{t}_ms"] = round(pc["total"], 3)
                row[f"uniform_{t}_gb"] = round(pc["memory"] / 1e9, 2)
        results.append(row)
    print(json.dumps({"config": a.config, "layers": a.layers, "gpus": a.gpus, "global_batch": a.global_batch, "degrees": degrees,
                      "comm": a.comm, "link_gbs": a.link_gbs,
                      "profile_ms": {str(t): {"fwd": prof[t]["f"], "bwd": prof[t]["b"], "workspace_gib": round(prof[t]["workspace"] / 2 ** 30, 2)}
                                     for t in degrees},
                      "plans": results}, indent=1))


if __name__ == "__main__":
    main()
