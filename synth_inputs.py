"""Seeded synthetic inputs shared by the CPU oracle tests and the HIP path.

This module holds no arithmetic of the method: it only draws random numbers,
rounds the bf16-stored tensors to bf16-representable values (so both sides
read bit-identical inputs) and slices the unsharded parameters of a layer
into one tensor-model-parallel rank's share (Megatron partition, Sec. II
"Tensor model parallelism": column split for QKV / FC1, row split for the
projection / FC2).

Workloads: GPT-style pre-LN layers at the hidden sizes of the paper's model
table (Table III), and LLaMA-style layers (RMSNorm, rotary embedding, SwiGLU); sequence length, head count and TP degree per config are
the ones this build is measured on.  Every tensor has its own
``numpy.random.default_rng([seed, layer, tensor_id])`` stream, so generation
order does not matter.
"""
from __future__ import annotations

import numpy as np

# name, hidden, heads, seq, batch, tp degree, sub-batches, layers, causal, dropout p, weight sigma
CONFIGS = {
    "C1": dict(hidden=512, n_heads=8, seq=128, batch=4, tp=2, n_sub=2, n_layers=1, causal=0, dropout_p=0.0, w_sigma=0.02),
    "C2": dict(hidden=1024, n_heads=16, seq=512, batch=8, tp=4, n_sub=2, n_layers=2, causal=1, dropout_p=0.1, w_sigma=0.02),
    "C3": dict(hidden=2048, n_heads=32, seq=1024, batch=8, tp=4, n_sub=2, n_layers=1, causal=1, dropout_p=0.1, w_sigma=0.02),
    "C4": dict(hidden=4096, n_heads=32, seq=2048, batch=4, tp=8, n_sub=2, n_layers=1, causal=1, dropout_p=0.1, w_sigma=0.02),
    "C5": dict(hidden=8192, n_heads=64, seq=2048, batch=2, tp=8, n_sub=4, n_layers=1, causal=1, dropout_p=0.1, w_sigma=0.01),
}

# Second layer family of the paper's model table (the LLaMA rows): pre-RMSNorm, rotary embedding, SwiGLU FFN of inner
# width `ffn_hidden`, no biases.  L4 is LLaMA-7B's layer at the same sequence length, batch and TP degree as C4.
LLAMA_CONFIGS = {
    "L1": dict(arch="llama", hidden=256, n_heads=4, seq=128, batch=4, tp=2, n_sub=2, n_layers=1, causal=1, dropout_p=0.0,
               ffn_hidden=704, rope_theta=10000.0, w_sigma=0.03),
    "L2": dict(arch="llama", hidden=1024, n_heads=16, seq=512, batch=4, tp=4, n_sub=2, n_layers=2, causal=1, dropout_p=0.1,
               ffn_hidden=2816, rope_theta=10000.0, w_sigma=0.02),
    "L4": dict(arch="llama", hidden=4096, n_heads=32, seq=2048, batch=4, tp=8, n_sub=2, n_layers=1, causal=1, dropout_p=0.0,
               ffn_hidden=11008, rope_theta=10000.0, w_sigma=0.02),
}

PARAM_NAMES = ("ln1_g", "ln1_b", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo",
               "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
_TENSOR_ID = {n: i for i, n in enumerate(PARAM_NAMES)}
_TENSOR_ID.update(x=100, dy=101, wg=50, wu=51)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable value (ties to even); result stays fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def _normal(seed, layer, name, shape, sigma, mean=0.0):
    rng = np.random.default_rng([int(seed), int(layer), _TENSOR_ID[name]])
    return (mean + sigma * rng.standard_normal(shape, dtype=np.float32)).astype(np.float32)


def make_layer_params(cfg: dict, layer: int, seed: int = 0) -> dict:
    """Unsharded parameters of one layer.  Matrices are [in, out] row-major and bf16-representable;
    biases and LayerNorm parameters are plain fp32."""
    h = cfg["hidden"]
    sw = cfg.get("w_sigma", 0.02)
    p = {}
    for name, shape in (("wq", (h, h)), ("wk", (h, h)), ("wv", (h, h)), ("wo", (h, h)),
                        ("w1", (h, 4 * h)), ("w2", (4 * h, h))):
        p[name] = round_to_bf16(_normal(seed, layer, name, shape, sw))
    for name, n in (("bq", h), ("bk", h), ("bv", h), ("bo", h), ("b1", 4 * h), ("b2", h),
                    ("ln1_b", h), ("ln2_b", h)):
        p[name] = _normal(seed, layer, name, (n,), 0.02)
    for name in ("ln1_g", "ln2_g"):
        p[name] = _normal(seed, layer, name, (h,), 0.02, mean=1.0)
    return p


def make_llama_layer_params(cfg: dict, layer: int, seed: int = 0) -> dict:
    """Unsharded parameters of one LLaMA-style layer: wq, wk, wv, wo [h,h], wg, wu [h,F], w2 [F,h] (bf16-representable),
    RMSNorm weights ln1_g, ln2_g [h] fp32."""
    h, F = cfg["hidden"], cfg["ffn_hidden"]
    sw = cfg.get("w_sigma", 0.02)
    p = {}
    for name, shape in (("wq", (h, h)), ("wk", (h, h)), ("wv", (h, h)), ("wo", (h, h)), ("wg", (h, F)), ("wu", (h, F)), ("w2", (F, h))):
        p[name] = round_to_bf16(_normal(seed, layer, name, shape, sw))
    for name in ("ln1_g", "ln2_g"):
        p[name] = _normal(seed, layer, name, (h,), 0.02, mean=1.0)
    return p


def shard_llama_layer_params(p: dict, cfg: dict, rank: int) -> dict:
    """Rank `rank`'s share: contiguous heads -> columns of wq/wk/wv and rows of wo; FFN columns
    [rank*F/t, (rank+1)*F/t) -> columns of wg, wu and rows of w2.  RMSNorm weights are replicated."""
    h, t, F = cfg["hidden"], cfg["tp"], cfg["ffn_hidden"]
    hp, fp = h // t, F // t
    a, f = slice(rank * hp, (rank + 1) * hp), slice(rank * fp, (rank + 1) * fp)
    s = {k: p[k] for k in ("ln1_g", "ln2_g")}
    for k in ("wq", "wk", "wv"):
        s[k] = np.ascontiguousarray(p[k][:, a])
    s["wo"] = np.ascontiguousarray(p["wo"][a, :])
    for k in ("wg", "wu"):
        s[k] = np.ascontiguousarray(p[k][:, f])
    s["w2"] = np.ascontiguousarray(p["w2"][f, :])
    return s


def make_activations(cfg: dict, seed: int = 0):
    """Layer input x and upstream gradient dy, [batch*seq, hidden] (batch-major token rows),
    N(0,1) rounded to bf16-representable fp32."""
    M, h = cfg["batch"] * cfg["seq"], cfg["hidden"]
    x = round_to_bf16(_normal(seed, 0, "x", (M, h), 1.0))
    dy = round_to_bf16(_normal(seed, 0, "dy", (M, h), 1.0))
    return x, dy


def shard_layer_params(p: dict, cfg: dict, rank: int) -> dict:
    """Rank `rank`'s share: contiguous heads [rank*nh/t, (rank+1)*nh/t) -> columns of wq/wk/wv and rows
    of wo; FFN columns [rank*4h/t, (rank+1)*4h/t) -> columns of w1 and rows of w2.  Replicated: LayerNorm
    parameters and the row-parallel biases bo, b2 (added once, after the reduction)."""
    h, t = cfg["hidden"], cfg["tp"]
    hp, fp = h // t, 4 * h // t
    a, f = slice(rank * hp, (rank + 1) * hp), slice(rank * fp, (rank + 1) * fp)
    s = {k: p[k] for k in ("ln1_g", "ln1_b", "ln2_g", "ln2_b", "bo", "b2")}
    for k in ("wq", "wk", "wv"):
        s[k] = np.ascontiguousarray(p[k][:, a])
    for k in ("bq", "bk", "bv"):
        s[k] = np.ascontiguousarray(p[k][a])
    s["wo"] = np.ascontiguousarray(p["wo"][a, :])
    s["w1"] = np.ascontiguousarray(p["w1"][:, f])
    s["b1"] = np.ascontiguousarray(p["b1"][f])
    s["w2"] = np.ascontiguousarray(p["w2"][f, :])
    return s


def small_config(**over) -> dict:
    """A tiny layer for brute-force checks (finite differences, hand-sized cases)."""
    c = dict(hidden=16, n_heads=2, seq=4, batch=2, tp=1, n_sub=1, n_layers=1, causal=1, dropout_p=0.0, w_sigma=0.2)
    c.update(over)
    return c
