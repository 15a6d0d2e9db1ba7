#!/usr/bin/env python3
"""Benchmark of the hot path: one TMP rank's transformer-layer shard, forward + backward, under the
sub-batch schedule, on ONE MI355X.  Prints one JSON line.

A step = one oases_forward + one oases_backward over one synthetic batch (inputs resident in HBM).
Metric: model TFLOP/s of the shard (GEMMs 2mnk, attention 2*M*s*hp causal / 4*M*s*hp full in forward,
backward = 2x forward; the score recomputation of the attention backward is not counted).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6     # MI355X dense bf16 MFMA (256 CU x 2.4 GHz x 4096 flop/clk/CU)
PEAK_HBM_GBS = 8000.0


def widths(cfg):
    """(hp, fp, fw): local attention width, local FFN inner width, columns of the FC1 GEMM (SwiGLU: gate and up)."""
    h, t = cfg["hidden"], cfg["tp"]
    llama = cfg.get("arch") == "llama"
    fp = (cfg["ffn_hidden"] if llama else 4 * h) // t
    return h // t, fp, (2 * fp if llama else fp)


def model_flops(cfg):
    M, h, s, t, L = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["seq"], cfg["tp"], cfg["n_layers"]
    hp, fp, fw = widths(cfg)
    gemm = 2.0 * M * h * (3 * hp + hp + fw + fp)
    attn = (2.0 if cfg["causal"] else 4.0) * M * s * hp
    return 3.0 * (gemm + attn) * L


def op_flops(line, cfg):
    """Algorithmic flops of one scheduled GEMM / attention operator (one sub-batch); 0 for the HBM-bound ones."""
    M, h, s, t = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["seq"], cfg["tp"]
    Ms = M if line.endswith("sb*") else M // cfg["n_sub"]
    hp, fp, fw = widths(cfg)
    op = line.split()[1]
    if op == "PROJ+QKV.wgrad":
        return 2.0 * Ms * h * (hp + 3 * hp)
    base = op.split(".")[0].split("+")[0]
    table = {"QKV": 2.0 * Ms * h * 3 * hp, "PROJ": 2.0 * Ms * hp * h, "FC1": 2.0 * Ms * h * fw, "FC2": 2.0 * Ms * fp * h}
    if base in table:
        return table[base]
    if base == "ATTN":
        f = (2.0 if cfg["causal"] else 4.0) * Ms * s * hp
        return 2.0 * f if op.endswith(".b") else f
    return 0.0


def op_bytes(line, cfg):
    """Algorithmic HBM bytes of one HBM-bound operator (one sub-batch): each tensor read once, written once."""
    M, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
    e = (M // cfg["n_sub"]) * h
    op = line.split()[1]
    per_elem = {"LN1": 4 + 2, "R1+BDR1+LN2": 4 + 4 + 4 + 2, "R2+BDR2": 4 + 4 + 4, "BDR2.b": 4 + 2,
                "R3+LN2.b+BDR1.b": 4 + 4 + 4 + 4 + 2, "R4+LN1.b": 4 + 4 + 4 + 4,
                "RMS1": 4 + 2, "R1+DR1+RMS2": 4 + 4 + 4 + 2, "R2+DR2": 4 + 4 + 4, "DR2.b": 4 + 2,
                "R3+RMS2.b+DR1.b": 4 + 4 + 4 + 4 + 2, "R4+RMS1.b": 4 + 4 + 4 + 4}
    if op.startswith("ROPE") and op != "ROPE.table":      # Q and K parts of the bf16 qkv rows, read and written
        return float((M // cfg["n_sub"]) * 2 * widths(cfg)[0] * 2 * 2)
    return float(per_elem.get(op, 0)) * e


def gemm_kernel_label(line, cfg, B, ws_bytes):
    """Kernel instantiation a GEMM operator runs on: (contraction form, epilogue, block tile)."""
    M, h, t = cfg["batch"] * cfg["seq"], cfg["hidden"], cfg["tp"]
    Ms = M if line.endswith("sb*") else M // cfg["n_sub"]
    hp, fp, fw = widths(cfg)
    llama = cfg.get("arch") == "llama"
    op = line.split()[1]
    if op.endswith(".r"):
        op = op[:-2]
    shapes = {"QKV": ("NN", "bf16" if llama else "bias_bf16", Ms, 3 * hp, h), "PROJ": ("NN", "f32", Ms, h, hp),
              "FC1+GELU": ("NN", "bias_gelu", Ms, fp, h), "FC1+SWIGLU": ("NN", "swiglu", Ms, fw, h),
              "FC2": ("NN", "f32", Ms, h, fp), "FC2.dgrad+dGELU": ("NT", "dgelu", Ms, fp, h), "FC2.dgrad+dSWIGLU": ("NT", "dswiglu", Ms, fp, h),
              "FC1.dgrad": ("NT", "f32", Ms, h, fw),
              "PROJ.dgrad": ("NT", "bf16", Ms, hp, h), "QKV.dgrad": ("NT", "f32", Ms, h, 3 * hp), "FC2.wgrad": ("TN", "acc_f32", fp, h, Ms),
              "FC1.wgrad": ("TN", "acc_f32", h, fw, Ms), "PROJ.wgrad": ("TN", "acc_f32", hp, h, Ms), "QKV.wgrad": ("TN", "acc_f32", h, 3 * hp, Ms)}
    if op == "PROJ+QKV.wgrad":   # the two weight gradients of the attention block in one launch
        return "gemm_TN_acc_f32_128x256_pp_pair"
    if op not in shapes:
        return None
    form, epi, m, n, k = shapes[op]
    epi_id = {"f32": 0, "bf16": 1, "bias_bf16": 2, "bias_gelu": 3, "dgelu": 4, "acc_f32": 0, "swiglu": 6, "dswiglu": 7}[epi]
    tile = B.lib.oases_op_gemm_variant({"NN": 0, "NT": 1, "TN": 2}[form], epi_id, m, n, k, ws_bytes)
    slices = tile // 1000000 % 100
    split = f"_splitk{slices}" if slices >= 2 else ""
    wk = "_pp" if tile >= 300000000 else "_dtl" if tile >= 200000000 else "_wavek2" if tile >= 100000000 else ""
    return f"gemm_{form}_{epi}_{tile // 1000 % 1000}x{tile % 1000}{wk}{split}"


def cpu_baseline(cfg, name):
    """The oracle as it stands, timed on the host cores: the rank-0 shard's layer (the same work the GPU does)."""
    import torch
    import synth_inputs as si
    if cfg.get("arch") == "llama":
        from oracle import llama_oracle as lo
        layers = [si.shard_llama_layer_params(si.make_llama_layer_params(cfg, l, 0), cfg, 0) for l in range(cfg["n_layers"])]
    else:
        from oracle import layer_oracle as lo
        layers = [si.shard_layer_params(si.make_layer_params(cfg, l, 0), cfg, 0) for l in range(cfg["n_layers"])]
    x, dy = si.make_activations(cfg, 0)
    reps, dt = 0, 0.0
    while reps == 0 or (dt < 10.0 and reps < 8):  # about 10 s of CPU work, at least one whole step
        t0 = time.perf_counter()
        lo.model_forward_backward(layers, x, dy, cfg, seed=0, dtype=torch.float32)
        dt += time.perf_counter() - t0
        reps += 1
    return {"value": round(reps * model_flops(cfg) / dt / 1e12, 4), "unit": "TFLOP/s", "cores": torch.get_num_threads(), "kind": "oracle",
            "seconds": round(dt, 2),
            "sample": f"the whole step: rank-0 shard of {name}, forward+backward, fp32 torch-CPU oracle, {reps} repetition(s)"}


class Workload:
    """Device-resident inputs, parameters, gradients and workspace of one rank-0 shard."""

    def __init__(self, name, n_sub=None, attn_dropout=None):
        import torch
        import synth_inputs as si
        from paper_2305_16121_amd import binding as B
        self.name = name
        cfg = dict({**si.CONFIGS, **si.LLAMA_CONFIGS}[name])
        if n_sub:
            cfg["n_sub"] = n_sub
        if attn_dropout is not None:
            cfg["attn_dropout_p"] = attn_dropout
        self.cfg = cfg
        x, dy = si.make_activations(cfg, 0)
        if cfg.get("arch") == "llama":
            self.W = [B.pack_llama_rank_params(si.shard_llama_layer_params(si.make_llama_layer_params(cfg, l, 0), cfg, 0)) for l in range(cfg["n_layers"])]
        else:
            self.W = [B.pack_rank_params(si.shard_layer_params(si.make_layer_params(cfg, l, 0), cfg, 0)) for l in range(cfg["n_layers"])]
        self.G = [B.zero_grads_like(w) for w in self.W]
        self.xd, self.dyd = torch.from_numpy(x).cuda(), torch.from_numpy(dy).cuda()
        self.yd, self.dxd = torch.empty_like(self.xd), torch.empty_like(self.xd)
        self.s1, self.s2 = torch.cuda.Stream(), torch.cuda.Stream()
        self.ws = None
        self.peers = None

    def handle(self, flags=0, n_sub=None):
        import torch
        from paper_2305_16121_amd import binding as B
        H = B.Handle(B.make_cfg(self.cfg, rank=0, seed=0, flags=flags, n_sub=n_sub))
        if self.ws is None or self.ws.numel() < H.workspace_bytes:
            self.ws = torch.empty(H.workspace_bytes, dtype=torch.uint8, device="cuda")
        return H

    def make_peers(self):
        """Peer sums at the four reduction points of every layer (any values: what is timed is the read beside the partial)."""
        import torch
        if self.peers is None:
            self.peers = [{k: 0.01 * torch.randn_like(self.xd) for k in ("fwd_attn", "fwd_ffn", "bwd_ffn", "bwd_attn")} for _ in self.W]
        return self.peers

    def step(self, H, peers=None):
        H.forward(self.W, self.xd, self.yd, self.ws, peers=peers, s_compute=self.s1, s_comm=self.s2)
        H.backward(self.W, self.xd, self.dyd, self.dxd, self.G, self.ws, peers=peers, s_compute=self.s1, s_comm=self.s2)

    def time_ms(self, H, steps, warmup, peers=None):
        import torch
        for _ in range(warmup):
            self.step(H, peers)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step(H, peers)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3


def mfma_rate(B):
    """Sustained rate of a register-resident MFMA loop (no memory traffic) with zero and with pseudo-random operands."""
    import torch
    wgs, iters = 1024, 4000
    out = torch.empty(wgs * 256, dtype=torch.float32, device="cuda")
    res = {}
    for label, rnd in (("zero_operands", 0), ("random_operands", 1)):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        st = torch.cuda.current_stream()
        for _ in range(2):
            B.check(B.lib.oases_probe_mfma_rate(rnd, iters, wgs, out.data_ptr(), st.cuda_stream))
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            B.check(B.lib.oases_probe_mfma_rate(rnd, iters, wgs, out.data_ptr(), st.cuda_stream))
        e1.record()
        torch.cuda.synchronize()
        res[label] = round(5 * wgs * 4 * iters * 8 * 32768.0 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    res["unit"] = "TFLOP/s"
    return res


def lds_load_rate(B):
    """Per-CU rate of L2-resident direct-to-LDS loads, one workgroup of four or eight waves per CU (GB/s per CU)."""
    import torch
    wgs, iters = 256, 4000
    src = torch.zeros(wgs * 65536, dtype=torch.uint8, device="cuda")
    out = torch.zeros(512, dtype=torch.float32, device="cuda")
    res = {}
    st = torch.cuda.current_stream()
    for waves in (4, 8):
        call = lambda: B.check(B.lib.oases_probe_lds_load_rate(waves, iters, wgs, src.data_ptr(), src.numel(), out.data_ptr(), st.cuda_stream))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        call()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(3):
            call()
        e1.record()
        torch.cuda.synchronize()
        res[f"{waves}_waves"] = round(3 * waves * iters * 8192.0 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
    res["unit"] = "GB/s per CU"
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="C4", help="workload: C1..C5 GPT layers (default C4, h=4096), L1/L2/L4 LLaMA-style layers")
    ap.add_argument("--n-sub", type=int, default=None, help="override the sub-batch count of the workload")
    ap.add_argument("--serialise", action="store_true", help="single stream")
    ap.add_argument("--recompute", action="store_true",
                    help="fine-grained recomputation: activations are rebuilt inside backward (model flops unchanged, more work)")
    ap.add_argument("--attn-dropout", type=float, default=None, help="dropout rate on the attention probabilities (off in the workloads)")
    ap.add_argument("--graph", action="store_true", help="capture one step into a HIP graph and time its replays (launch-bound small layers)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the further timings (one stream, n_sub = 1, peer sums, pinned kernels, C5, MFMA rate)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run one plain elementwise kernel of known size (reads and writes 256 MiB) first: the unit check for rocprofv3 byte counters")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no collectives, no sharding across GPUs); use --gpus 1")

    import torch
    import synth_inputs as si
    from paper_2305_16121_amd import binding as B
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    wl = Workload(a.config, a.n_sub, a.attn_dropout)
    cfg = wl.cfg
    M, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
    W, G, xd, dyd, yd, dxd, s1, s2 = wl.W, wl.G, wl.xd, wl.dyd, wl.yd, wl.dxd, wl.s1, wl.s2
    flags = (B.FLAG_SERIALISE if a.serialise else 0) | (B.FLAG_RECOMPUTE if a.recompute else 0)
    H = wl.handle(flags)
    step = wl.step

    if a.calib_copy:
        src = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        dst = src * 2.0          # one elementwise kernel: 256 MiB read, 256 MiB written
        torch.cuda.synchronize()
        del src, dst
    for _ in range(a.warmup):
        step(H)
    torch.cuda.synchronize()
    run = lambda: step(H)
    if a.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s1):
            step(H)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        run = graph.replay
    t0 = time.perf_counter()
    for _ in range(a.steps):
        run()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / a.steps
    flops = model_flops(cfg)
    tflops = flops / dt / 1e12

    out = {"metric": "model TFLOP/s of one TMP-rank layer shard, forward+backward, sub-batched (ms per step in ms_per_step)",
           "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
           "ms_per_step": round(dt * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic",
           "config": {"workload": f"{a.config}: {'LLaMA-style' if cfg.get('arch') == 'llama' else 'GPT'} layer h={h} heads={cfg['n_heads']} seq={cfg['seq']} batch={cfg['batch']} "
                                  f"t={cfg['tp']} rank 0 layers={cfg['n_layers']} causal={cfg['causal']} p={cfg['dropout_p']}" + (f" ffn={cfg['ffn_hidden']}" if cfg.get("arch") == "llama" else ""),
                      "n_sub": cfg["n_sub"], "attn_dropout_p": cfg.get("attn_dropout_p", 0.0), "streams": 1 if a.serialise else 2, "hip_graph": bool(a.graph), "recompute": bool(a.recompute),
                      "workspace_mib": round(H.workspace_bytes / 2 ** 20, 1), "model_gflop_per_step": round(flops / 1e9, 1),
                      "frac_of_bf16_peak": round(tflops / PEAK_BF16_TFLOPS, 4)}}

    # per-operator HIP-event timers over the same schedule (serialised so that every bracket holds one operator)
    if not a.no_profile:
        HP = wl.handle(B.FLAG_SERIALISE | B.FLAG_PROFILE | (B.FLAG_RECOMPUTE if a.recompute else 0))
        acc = {}
        reps = max(3, min(a.steps, 10))
        step(HP)
        for _ in range(reps):
            step(HP)
            torch.cuda.synchronize()
            for bwd in (False, True):
                for line, ms in HP.profile(bwd):
                    if " join " in line:
                        continue
                    lab = gemm_kernel_label(line, cfg, B, HP.gemm_workspace_bytes) or line.split()[1]
                    d = acc.setdefault(lab, dict(ms=0.0, launches=0, flops=0.0, bytes=0.0))
                    d["ms"] += ms
                    d["launches"] += 1
                    d["flops"] += op_flops(line, cfg)
                    d["bytes"] += op_bytes(line, cfg)
        table = []
        for lab, d in acc.items():
            avg_ms = d["ms"] / d["launches"]
            row = {"kernel": lab, "launches_per_step": d["launches"] // reps, "avg_ms": round(avg_ms, 4),
                   "ms_per_step": round(d["ms"] / reps, 4)}
            if d["flops"]:
                row["tflops"] = round(d["flops"] / d["launches"] / (avg_ms * 1e-3) / 1e12, 1)
                row["frac_of_mfma_peak"] = round(row["tflops"] / PEAK_BF16_TFLOPS, 3)
            if d["bytes"]:
                row["gbs"] = round(d["bytes"] / d["launches"] / (avg_ms * 1e-3) / 1e9, 1)
                row["frac_of_hbm_peak"] = round(row["gbs"] / PEAK_HBM_GBS, 3)
            table.append(row)
        table.sort(key=lambda r: -r["ms_per_step"])
        out["kernels"] = table
        out["config"]["serialised_sum_ms"] = round(sum(r["ms_per_step"] for r in table), 4)
        dom = next(r for r in table if r["kernel"].startswith("gemm_"))
        d = acc[dom["kernel"]]
        traffic = None     # HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, stored under profiles/
        tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
        if os.path.exists(tpath):
            traffic = json.load(open(tpath)).get(a.config, {}).get(dom["kernel"])
        out["roofline"] = {"kernel": dom["kernel"], "bound": "mfma", "achieved": dom["tflops"], "peak": PEAK_BF16_TFLOPS,
                           "unit": "TFLOP/s", "frac": round(dom["tflops"] / PEAK_BF16_TFLOPS, 4), "traffic": traffic,
                           "avg_launch_ms": dom["avg_ms"], "flops_per_launch": d["flops"] / d["launches"]}
        HP.close()

    # further measurements of the same build, each its own short timing (not part of `value`)
    if not a.no_extra:
        k, w = max(5, a.steps // 2), 3
        rflag = B.FLAG_RECOMPUTE if a.recompute else 0
        ex = {}
        ex["two_streams_ms"] = round(wl.time_ms(wl.handle(rflag), k, w), 4)
        ex["one_stream_ms"] = round(wl.time_ms(wl.handle(rflag | B.FLAG_SERIALISE), k, w), 4)
        ex["n_sub_1_ms"] = round(wl.time_ms(wl.handle(rflag, n_sub=1), k, w), 4)          # arithmetic-density loss of sub-batching (Fig. 5)
        ex["with_peer_sums_ms"] = round(wl.time_ms(wl.handle(rflag), k, w, peers=wl.make_peers()), 4)   # reduction points read a peer sum
        ex["pinned_kernel_choice_ms"] = round(wl.time_ms(wl.handle(rflag | B.FLAG_PIN_GEMM), k, w), 4)
        ex["mfma_rate_from_registers"] = mfma_rate(B)
        ex["direct_to_lds_load_rate"] = lds_load_rate(B)
        if a.config == "C4":          # the other configuration the target is quoted on
            w5 = Workload("C5")
            ms5 = w5.time_ms(w5.handle(0), k, w)
            f5 = model_flops(w5.cfg)
            ex["C5"] = {"workload": "C5: GPT layer h=8192 heads=64 seq=2048 batch=2 t=8 rank 0 causal p=0.1, n_sub=4, two streams",
                        "ms_per_step": round(ms5, 4), "tflops": round(f5 / ms5 / 1e9, 1), "frac_of_bf16_peak": round(f5 / ms5 / 1e9 / PEAK_BF16_TFLOPS, 4),
                        "one_stream_ms": round(w5.time_ms(w5.handle(B.FLAG_SERIALISE), k, w), 4),
                        "n_sub_1_ms": round(w5.time_ms(w5.handle(0, n_sub=1), k, w), 4)}
        out["extra"] = ex

    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, a.config)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
