"""ctypes binding of liboases.so: argument marshalling only (see include/oases.h for semantics)."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liboases.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} not built: run `python {os.path.join(_HERE, 'csrc', 'build.py')}` "
                      "(there is no CPU fallback for the HIP path)")
lib = C.CDLL(LIB_PATH)

OK, EINVAL, ENULL, EALIGN, EWORKSPACE, EHIP = 0, -1, -2, -3, -4, -5
GEMM_NN, GEMM_NT, GEMM_TN = 0, 1, 2
EPI_F32, EPI_BF16, EPI_BIAS_BF16, EPI_BIAS_GELU, EPI_DGELU = 0, 1, 2, 3, 4
EPI_SWIGLU, EPI_DSWIGLU = 6, 7
FLAG_SERIALISE, FLAG_PROFILE, FLAG_RECOMPUTE, FLAG_PIN_GEMM = 1, 2, 4, 8
ARCH_GPT, ARCH_LLAMA, ARCH_BERT = 0, 1, 2

_P = C.c_void_p
_PARAMS = ("ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo", "ln2_g", "ln2_b", "w1", "b1", "w2", "b2")
_PEERS = ("fwd_attn", "fwd_ffn", "bwd_ffn", "bwd_attn")


class LayerCfg(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_heads", C.c_int32), ("seq", C.c_int32), ("batch", C.c_int32),
                ("tp_degree", C.c_int32), ("tp_rank", C.c_int32), ("n_sub", C.c_int32), ("n_layers", C.c_int32),
                ("causal", C.c_int32), ("dropout_p", C.c_float), ("seed", C.c_uint64), ("ln_eps", C.c_float),
                ("flags", C.c_int32), ("arch", C.c_int32), ("ffn_hidden", C.c_int32), ("rope_theta", C.c_float), ("attn_dropout_p", C.c_float)]


class Weights(C.Structure):
    _fields_ = [(n, _P) for n in _PARAMS]


class Grads(C.Structure):
    _fields_ = [(n, _P) for n in _PARAMS]


class PeerSums(C.Structure):
    _fields_ = [(n, _P) for n in _PEERS]


def _sig(name, res, *args):
    f = getattr(lib, name)
    f.restype, f.argtypes = res, list(args)
    return f


_i, _f, _u64, _i64, _sz = C.c_int, C.c_float, C.c_uint64, C.c_int64, C.c_size_t
_sig("oases_last_error", C.c_char_p)
_sig("oases_create", _i, C.POINTER(LayerCfg), C.POINTER(_P))
_sig("oases_destroy", None, _P)
_sig("oases_workspace_bytes", _sz, _P)
_sig("oases_forward", _i, _P, C.POINTER(Weights), _P, _P, C.POINTER(PeerSums), _P, _sz, _P, _P)
_sig("oases_backward", _i, _P, C.POINTER(Weights), _P, _P, _P, C.POINTER(Grads), C.POINTER(PeerSums), _P, _sz, _P, _P)
_sig("oases_forward_segment", _i, _P, _i, _i, C.POINTER(Weights), _P, _P, _P, _sz, _P, _P, _P)
_sig("oases_backward_segment", _i, _P, _i, _i, C.POINTER(Weights), _P, _P, _P, C.POINTER(Grads), _P, _sz, _P, _P, _P)
_sig("oases_schedule_dump", _i, _P, _i, C.c_char_p, _sz)
_sig("oases_profile_read", _i, _P, _i, C.POINTER(C.c_float), _i)
_sig("oases_workspace_tensor", _i, _P, C.c_char_p, _i, C.POINTER(_sz), C.POINTER(_sz))
_sig("oases_op_dropout_mask", _i, _P, _u64, _i, _i, _i64, _i, _i, _f, _P)
_sig("oases_op_layernorm_fwd", _i, _P, _P, _P, _P, _P, _P, _i, _i, _f, _P)
_sig("oases_op_bias_dropout_residual_ln", _i, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _i, _i, _f, _u64, _i, _i, _i64, _f, _P)
_sig("oases_op_dropout_bwd", _i, _P, _P, _P, _i, _i, _u64, _i, _i, _i64, _f, _P, _P)
_sig("oases_op_layernorm_bwd", _i, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _P, _i, _i, _u64, _i, _i, _i64, _f, _P, _P)
_sig("oases_op_rmsnorm_fwd", _i, _P, _P, _P, _P, _i, _i, _f, _P)
_sig("oases_op_dropout_residual_rmsnorm", _i, _P, _P, _P, _P, _P, _P, _P, _i, _i, _f, _u64, _i, _i, _i64, _f, _P)
_sig("oases_op_rmsnorm_bwd", _i, _P, _P, _P, _P, _P, _P, _P, _P, _P, _i, _i, _u64, _i, _i, _i64, _f, _P, _P)
_sig("oases_op_rope_table", _i, _P, _i, _i, _f, _P)
_sig("oases_op_rope", _i, _P, _i, _i, _i64, _i, _i, _i, _P, _i, _P)
_sig("oases_op_gemm", _i, _i, _i, _i, _i, _i, _P, _i, _P, _i, _P, _i, _P, _P, _i, _P, _sz, _P)
_sig("oases_op_gemm_variant", _i, _i, _i, _i, _i, _i, _sz)
_sig("oases_op_gemm_tn_pair", _i, _i, _i, _i, _P, _i, _P, _i, _P, _i, _i, _i, _P, _i, _P, _i, _P, _i, _P)
_sig("oases_op_gemm_tn_pair_wins", _i, _i, _i, _i, _i, _i)
_sig("oases_op_gemm_forced", _i, _i, _i, _i, _i, _i, _i, _P, _i, _P, _i, _P, _i, _P, _P, _i, _P, _sz, _P)
_sig("oases_gemm_workspace_bytes", _sz, _P)
_sig("oases_op_colsum_bf16", _i, _P, _i, _i, _i, _P, _P, _P)
_sig("oases_op_colsum_bf16_static", _i, _P, _i, _i, _i, _P, _P)
_sig("oases_probe_mfma_rate", _i, _i, _i, _i, _P, _P)
_sig("oases_probe_lds_load_rate", _i, _i, _i, _i, _P, _sz, _P, _P)
_sig("oases_op_attention_fwd", _i, _P, _P, _P, _i, _i, _i, _i, _i, _i, _i, _P)
_sig("oases_op_attention_bwd", _i, _P, _P, _P, _P, _P, _P, _i, _i, _i, _i, _i, _i, _i, _P)
_sig("oases_op_attention_dropout_fwd", _i, _P, _P, _P, _i, _i, _i, _i, _i, _i, _i, _u64, _i, _f, _i, _i, _P)
_sig("oases_op_attention_dropout_bwd", _i, _P, _P, _P, _P, _P, _P, _i, _i, _i, _i, _i, _i, _i, _u64, _i, _f, _i, _i, _P)


class OasesError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"oases error {code}: {lib.oases_last_error().decode()}")


def check(rc):
    if rc != 0:
        raise OasesError(rc)


def ptr(t):
    """Device (or NULL) pointer of a torch tensor / raw int."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def nbytes(t):
    """Size in bytes of a torch tensor handed over as a buffer (0 for None)."""
    return 0 if t is None else t.numel() * t.element_size()


def stream_ptr(s):
    if s is None:
        return None
    return s if isinstance(s, int) else s.cuda_stream


def make_cfg(cfg: dict, rank: int = 0, seed: int = 0, flags: int = 0, n_sub: int | None = None) -> LayerCfg:
    llama = cfg.get("arch") == "llama"
    return LayerCfg(cfg["hidden"], cfg["n_heads"], cfg["seq"], cfg["batch"], cfg["tp"], rank,
                    cfg["n_sub"] if n_sub is None else n_sub, cfg["n_layers"], cfg["causal"], cfg["dropout_p"], seed,
                    0.0, flags, ARCH_LLAMA if llama else ARCH_BERT if cfg.get("arch") == "bert" else ARCH_GPT, cfg.get("ffn_hidden", 0) if llama else 0,
                    cfg.get("rope_theta", 0.0) if llama else 0.0, cfg.get("attn_dropout_p", 0.0))


class Handle:
    """Owns an oases_handle."""

    def __init__(self, c: LayerCfg):
        self.cfg = c
        h = _P()
        check(lib.oases_create(C.byref(c), C.byref(h)))
        self._h = h

    def close(self):
        if self._h:
            lib.oases_destroy(self._h)
            self._h = None

    __del__ = close

    @property
    def workspace_bytes(self) -> int:
        return lib.oases_workspace_bytes(self._h)

    @property
    def gemm_workspace_bytes(self) -> int:
        return lib.oases_gemm_workspace_bytes(self._h)

    def schedule(self, backward: bool) -> str:
        n = lib.oases_schedule_dump(self._h, int(backward), None, 0)
        buf = C.create_string_buffer(n + 1)
        lib.oases_schedule_dump(self._h, int(backward), buf, n + 1)
        return buf.value.decode()

    def profile(self, backward: bool):
        """[(operator line of the schedule, milliseconds)] of the last pass (needs FLAG_PROFILE)."""
        names = self.schedule(backward).strip().splitlines()
        ms = (C.c_float * len(names))()
        n = lib.oases_profile_read(self._h, int(backward), ms, len(names))
        if n < 0:
            raise OasesError(n)
        return list(zip(names, [float(v) for v in ms]))

    def tensor_span(self, name: str, layer: int = 0):
        off, nb = _sz(), _sz()
        check(lib.oases_workspace_tensor(self._h, name.encode(), layer, C.byref(off), C.byref(nb)))
        return off.value, nb.value

    @staticmethod
    def _structs(cls, names, dicts):
        arr = (cls * len(dicts))()
        for i, d in enumerate(dicts):
            for n in names:
                setattr(arr[i], n, ptr(d.get(n)) if d is not None else None)
        return arr

    def forward(self, weights, x, y, workspace, peers=None, s_compute=None, s_comm=None):
        w = self._structs(Weights, _PARAMS, weights)
        p = self._structs(PeerSums, _PEERS, peers) if peers is not None else None
        check(lib.oases_forward(self._h, w, ptr(x), ptr(y), p, ptr(workspace), nbytes(workspace), stream_ptr(s_compute), stream_ptr(s_comm)))

    def backward(self, weights, x, dy, dx, grads, workspace, peers=None, s_compute=None, s_comm=None):
        w = self._structs(Weights, _PARAMS, weights)
        g = self._structs(Grads, _PARAMS, grads)
        p = self._structs(PeerSums, _PEERS, peers) if peers is not None else None
        check(lib.oases_backward(self._h, w, ptr(x), ptr(dy), ptr(dx), g, p, ptr(workspace), nbytes(workspace), stream_ptr(s_compute),
                                 stream_ptr(s_comm)))


    def forward_segment(self, layer, segment, weights, x, y, workspace, partial_out=None, reduced_in=None, stream=None):
        w = self._structs(Weights, _PARAMS, weights)
        check(lib.oases_forward_segment(self._h, layer, segment, w, ptr(x), ptr(y), ptr(workspace), nbytes(workspace), ptr(partial_out), ptr(reduced_in),
                                        stream_ptr(stream)))

    def backward_segment(self, layer, segment, weights, x, dy, dx, grads, workspace, partial_out=None, reduced_in=None, stream=None):
        w = self._structs(Weights, _PARAMS, weights)
        g = self._structs(Grads, _PARAMS, grads)
        check(lib.oases_backward_segment(self._h, layer, segment, w, ptr(x), ptr(dy), ptr(dx), g, ptr(workspace), nbytes(workspace), ptr(partial_out),
                                         ptr(reduced_in), stream_ptr(stream)))


# ------------------------------------------------------------------------------------------------
# device-side layout of one rank's parameters (marshalling only)
# ------------------------------------------------------------------------------------------------
def pack_rank_params(shard: dict, device="cuda"):
    """numpy dict from synth_inputs.shard_layer_params -> dict of device tensors in the library's layout:
    wqkv [h,3hp] = [wq | wk | wv] bf16, bqkv [3hp] fp32, the other matrices bf16, vectors fp32."""
    import numpy as np
    import torch
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dt)
    out = {
        "wqkv": t(np.concatenate([shard["wq"], shard["wk"], shard["wv"]], axis=1), torch.bfloat16),
        "bqkv": t(np.concatenate([shard["bq"], shard["bk"], shard["bv"]]), torch.float32),
    }
    for k in ("wo", "w1", "w2"):
        out[k] = t(shard[k], torch.bfloat16)
    for k in ("ln1_g", "ln1_b", "bo", "ln2_g", "ln2_b", "b1", "b2"):
        out[k] = t(shard[k], torch.float32)
    return out


def interleave_gate_up(gate, up):
    """[.., fp] x 2 -> [.., 2fp]: blocks of 32 gate columns, each followed by the same 32 up columns (the layout of
    w1 and of the stored pre-activations in the LLaMA-style layer, see OASES_ARCH_LLAMA)."""
    import numpy as np
    *lead, fp = gate.shape
    return np.stack([gate.reshape(*lead, fp // 32, 32), up.reshape(*lead, fp // 32, 32)], axis=-2).reshape(*lead, 2 * fp)


def split_gate_up(w13):
    """Inverse of interleave_gate_up on a numpy array or torch tensor: [.., 2fp] -> (gate [.., fp], up [.., fp])."""
    *lead, two_fp = w13.shape
    v = w13.reshape(*lead, two_fp // 64, 2, 32)
    return v[..., 0, :].reshape(*lead, two_fp // 2), v[..., 1, :].reshape(*lead, two_fp // 2)


def pack_llama_rank_params(shard: dict, device="cuda"):
    """numpy dict from synth_inputs.shard_llama_layer_params -> device tensors in the library's layout: wqkv [h,3hp],
    w1 [h,2fp] = gate / up columns interleaved in blocks of 32, wo, w2 bf16; RMSNorm weights fp32."""
    import numpy as np
    import torch
    t = lambda a, dt: torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=dt)
    return {"wqkv": t(np.concatenate([shard["wq"], shard["wk"], shard["wv"]], axis=1), torch.bfloat16),
            "w1": t(interleave_gate_up(shard["wg"], shard["wu"]), torch.bfloat16),
            "wo": t(shard["wo"], torch.bfloat16), "w2": t(shard["w2"], torch.bfloat16),
            "ln1_g": t(shard["ln1_g"], torch.float32), "ln2_g": t(shard["ln2_g"], torch.float32)}


def zero_grads_like(params: dict):
    import torch
    return {k: torch.zeros(v.shape, dtype=torch.float32, device=v.device) for k, v in params.items()}
