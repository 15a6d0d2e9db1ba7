"""Shared helpers of the GPU parity tests."""
import numpy as np
import torch


def rel_err(got, ref):
    """The contract's metric: max|got - ref| / rms(ref)."""
    got = torch.as_tensor(got).detach().double().cpu()
    ref = torch.as_tensor(ref).detach().double().cpu()
    rms = float(torch.sqrt((ref ** 2).mean()))
    return float((got - ref).abs().max()) / max(rms, 1e-30)


def rms_err(got, ref):
    got = torch.as_tensor(got).detach().double().cpu()
    ref = torch.as_tensor(ref).detach().double().cpu()
    return float(torch.sqrt(((got - ref) ** 2).mean())) / max(float(torch.sqrt((ref ** 2).mean())), 1e-30)


def bf16_round(t):
    return t.to(torch.bfloat16).to(t.dtype)


def dev(a, dtype=None):
    t = torch.as_tensor(np.ascontiguousarray(a) if isinstance(a, np.ndarray) else a)
    return t.to(device="cuda", dtype=dtype or t.dtype).contiguous()


def randn(gen, *shape, scale=1.0):
    return (scale * torch.randn(*shape, generator=gen, dtype=torch.float64))


def bf16_close(got, ref, extra_rel=0.0, extra_abs=0.0):
    """Checks `got` (values that went through one bf16 rounding) against `ref`: every element within half a
    bf16 ulp of the reference plus an allowance extra_rel*|ref| + extra_abs for the arithmetic in front of
    the rounding.  Returns (ok, message)."""
    got = torch.as_tensor(got).detach().double().cpu()
    ref = torch.as_tensor(ref).detach().double().cpu()
    mag = ref.abs().clamp_min(1e-30)
    ulp = torch.pow(2.0, torch.floor(torch.log2(mag)) - 7)
    tol = 0.5 * ulp + extra_rel * mag + extra_abs + 1e-30
    excess = (got - ref).abs() - tol
    nbad = int((excess > 0).sum())
    if nbad == 0:
        return True, ""
    i = int(torch.argmax(excess))
    return False, (f"{nbad}/{got.numel()} elements beyond half a bf16 ulp; worst at flat index {i}: got "
                   f"{float(got.flatten()[i])!r} ref {float(ref.flatten()[i])!r} ulp {float(ulp.flatten()[i])!r}")


def assert_bf16_close(got, ref, extra_rel=0.0, extra_abs=0.0, what=""):
    ok, msg = bf16_close(got, ref, extra_rel, extra_abs)
    assert ok, f"{what} {msg}"
