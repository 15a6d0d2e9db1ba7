"""Per-operator parity of the kernels of the LLaMA-style layer (RMSNorm forward / fused / backward, rotary embedding,
SwiGLU epilogues of the GEMM) against the oracle's operator definitions, through the C ABI."""
import numpy as np
import pytest
import torch

from tests.util import rel_err, bf16_round, assert_bf16_close, dev, randn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_16121_amd import binding
    return binding


@pytest.fixture(scope="module")
def ll():
    from oracle import llama_oracle
    return llama_oracle


@pytest.fixture(scope="module")
def lo():
    from oracle import layer_oracle
    return layer_oracle


def gen(seed):
    g = torch.Generator()
    g.manual_seed(seed)
    return g


@pytest.mark.parametrize("rows,h", [(300, 512), (70, 1000), (33, 4096), (9, 8192), (5, 11008), (4, 8)])
def test_rmsnorm_fwd(B, ll, rows, h):
    g = gen(1)
    x = randn(g, rows, h) * 3 + 0.5
    gam = 1 + 0.1 * randn(g, h)
    xd, gd = dev(x, torch.float32), dev(gam, torch.float32)
    out = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    rstd = torch.empty(rows, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_rmsnorm_fwd(xd.data_ptr(), gd.data_ptr(), out.data_ptr(), rstd.data_ptr(), rows, h, 1e-5, None))
    ref, rr = ll.rms_norm_fwd(xd.cpu().double(), gd.cpu().double(), 1e-5)
    assert_bf16_close(out.float(), ref, 1e-5, 2e-6 * float(ref.abs().max()))
    assert rel_err(rstd, rr.flatten()) < 1e-5


@pytest.mark.parametrize("rows,h,p,with_peer,with_ln", [(130, 512, 0.1, True, True), (33, 1000, 0.0, False, True), (17, 4096, 0.5, True, False)])
def test_dropout_residual_rmsnorm(B, ll, lo, rows, h, p, with_peer, with_ln):
    g = gen(2)
    part, peer, xin = randn(g, rows, h), randn(g, rows, h), randn(g, rows, h)
    gam = 1 + 0.1 * randn(g, h)
    d = {k: dev(v, torch.float32) for k, v in dict(part=part, peer=peer, xin=xin, gam=gam).items()}
    c = {k: v.cpu().double() for k, v in d.items()}
    xo = torch.empty(rows, h, dtype=torch.float32, device="cuda")
    out = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    rstd = torch.empty(rows, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_dropout_residual_rmsnorm(d["part"].data_ptr(), d["peer"].data_ptr() if with_peer else None, d["xin"].data_ptr(),
                                                    xo.data_ptr(), d["gam"].data_ptr() if with_ln else None,
                                                    out.data_ptr() if with_ln else None, rstd.data_ptr() if with_ln else None, rows, h, 1e-5,
                                                    77, 2, 1, 640, p, None))
    keep = torch.from_numpy(lo.dropout_keep_mask(77, 2, 1, rows, h, p, row0=640)).double()
    rxo = c["xin"] + keep * (c["part"] + (c["peer"] if with_peer else 0)) / (1 - p)
    assert rel_err(xo, rxo) < 1e-6
    if with_ln:
        ref, rr = ll.rms_norm_fwd(xo.cpu().double(), c["gam"], 1e-5)
        assert_bf16_close(out.float(), ref, 1e-5, 2e-6 * float(ref.abs().max()))
        assert rel_err(rstd, rr.flatten()) < 1e-5


@pytest.mark.parametrize("rows,h,p,with_peer,with_dz", [(300, 512, 0.1, True, True), (70, 1000, 0.0, False, False), (40, 4096, 0.5, True, True),
                                                        (2100, 4096, 0.0, False, True)])
def test_rmsnorm_bwd(B, ll, lo, rows, h, p, with_peer, with_dz):
    g = gen(4)
    part, peer, dres, x = randn(g, rows, h), randn(g, rows, h), randn(g, rows, h), randn(g, rows, h) * 2 + 1
    gam = 1 + 0.1 * randn(g, h)
    d = {k: dev(v, torch.float32) for k, v in dict(part=part, peer=peer, dres=dres, x=x, gam=gam).items()}
    c = {k: v.cpu().double() for k, v in d.items()}
    _, rr = ll.rms_norm_fwd(c["x"], c["gam"], 1e-5)
    rstd = dev(rr.flatten(), torch.float32)
    dxo = torch.empty(rows, h, dtype=torch.float32, device="cuda")
    dz = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    dgam = torch.full((h,), 0.5, dtype=torch.float32, device="cuda")
    scratch = torch.full((3 * 1024 * h,), float("nan"), dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_rmsnorm_bwd(d["part"].data_ptr(), d["peer"].data_ptr() if with_peer else None, d["dres"].data_ptr(),
                                       d["x"].data_ptr(), rstd.data_ptr(), d["gam"].data_ptr(), dxo.data_ptr(), dgam.data_ptr(),
                                       dz.data_ptr() if with_dz else None, rows, h, 9, 0, 1, 128, p, scratch.data_ptr(), None))
    gin = c["part"] + (c["peer"] if with_peer else 0)
    rdx, rdg = ll.rms_norm_bwd(gin, c["x"], rstd.cpu().double()[:, None], c["gam"])
    ref = c["dres"] + rdx
    assert rel_err(dxo, ref) < 2e-5
    assert rel_err(dgam, rdg + 0.5) < 2e-5                  # accumulated into
    if with_dz:
        keep = torch.from_numpy(lo.dropout_keep_mask(9, 0, 1, rows, h, p, row0=128)).double()
        rz = keep * ref / (1 - p)
        assert_bf16_close(dz.float(), rz, 1e-5, 2e-6 * float(rz.abs().max()))


@pytest.mark.parametrize("batch,seq,heads,d,row0,rows", [(2, 96, 3, 64, 0, 192), (3, 200, 2, 128, 200, 264), (1, 2048, 1, 128, 1900, 148)])
def test_rope(B, ll, batch, seq, heads, d, row0, rows):
    """Table against fp64 angles; rotation of a row range (positions wrap at sequence ends) and its inverse."""
    tab = torch.empty(seq, d // 2, 2, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_rope_table(tab.data_ptr(), seq, d, 10000.0, None))
    ang = ll.rope_angles(seq, d, 10000.0, torch.float64)
    assert float((tab[..., 0].cpu().double() - torch.cos(ang)).abs().max()) < 1e-7
    assert float((tab[..., 1].cpu().double() - torch.sin(ang)).abs().max()) < 1e-7
    hp = heads * d
    M = batch * seq
    g = gen(5)
    qkv = bf16_round(randn(g, M, 3 * hp))
    qd = dev(qkv, torch.bfloat16)
    B.check(B.lib.oases_op_rope(qd[row0:].data_ptr(), 3 * hp, rows, row0, seq, heads, d, tab.data_ptr(), 0, None))
    ref = qkv.double().clone()
    for part in (0, 1):
        ref[:, part * hp:(part + 1) * hp] = ll.rope_apply(qkv.double()[:, part * hp:(part + 1) * hp], batch, seq, d, 10000.0)
    got = qd.float().cpu().double()
    assert torch.equal(got[:row0], qkv.double()[:row0]) and torch.equal(got[row0 + rows:], qkv.double()[row0 + rows:])   # rows outside untouched
    assert torch.equal(got[:, 2 * hp:], qkv.double()[:, 2 * hp:])                                                           # V untouched
    assert_bf16_close(got[row0:row0 + rows, :2 * hp].float(), ref[row0:row0 + rows, :2 * hp], 1e-5, 1e-5)
    # inverse rotation of the rotated values: the original up to two bf16 roundings
    B.check(B.lib.oases_op_rope(qd[row0:].data_ptr(), 3 * hp, rows, row0, seq, heads, d, tab.data_ptr(), 1, None))
    back = ll.rope_apply(got[:, :hp], batch, seq, d, 10000.0, inverse=True)
    assert_bf16_close(qd.float().cpu()[row0:row0 + rows, :hp], back[row0:row0 + rows], 1e-5, 1e-5)


def interleave(gate, up):
    """[.., fp] x 2 -> [.., 2 fp]: blocks of 32 gate columns followed by the same 32 up columns."""
    *lead, fp = gate.shape
    return torch.stack([gate.reshape(*lead, fp // 32, 32), up.reshape(*lead, fp // 32, 32)], dim=-2).reshape(*lead, 2 * fp)


@pytest.mark.parametrize("M,fp,K", [(384, 352, 256), (136, 96, 72), (1032, 1376, 520)])
@pytest.mark.parametrize("variant", [0, 1256256, 1128256, 101128256, 101256128, 1128128])
def test_gemm_swiglu_epilogues(B, ll, M, fp, K, variant):
    g = gen(7)
    a = bf16_round(randn(g, M, K))
    wg, wu = bf16_round(randn(g, K, fp, scale=0.05)), bf16_round(randn(g, K, fp, scale=0.05))
    w13 = interleave(wg, wu)
    ad, wd = dev(a, torch.bfloat16), dev(w13, torch.bfloat16)
    f = torch.empty(M, fp, dtype=torch.bfloat16, device="cuda")
    gu = torch.empty(M, 2 * fp, dtype=torch.bfloat16, device="cuda")
    if variant:
        B.check(B.lib.oases_op_gemm_forced(variant, B.GEMM_NN, B.EPI_SWIGLU, M, 2 * fp, K, ad.data_ptr(), K, wd.data_ptr(), 2 * fp, f.data_ptr(), fp,
                                           None, gu.data_ptr(), 2 * fp, None, 0, None))
    else:
        B.check(B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_SWIGLU, M, 2 * fp, K, ad.data_ptr(), K, wd.data_ptr(), 2 * fp, f.data_ptr(), fp,
                                    None, gu.data_ptr(), 2 * fp, None, 0, None))
    gate, up = a.double() @ wg.double(), a.double() @ wu.double()
    assert_bf16_close(gu.float(), interleave(gate, up), 1e-5, 2e-6 * float(gate.abs().max()))
    assert_bf16_close(f.float(), ll.silu(gate) * up, 1e-4, 1e-5)
    # gradient epilogue on the input-gradient form: dF = dZ W2^T, then [dgate | dup]
    dz = bf16_round(randn(g, M, K))
    w2 = bf16_round(randn(g, fp, K, scale=0.05))                 # [fp, h]: dF = dz @ w2^T is the NT form with B = w2
    dzd, w2d = dev(dz, torch.bfloat16), dev(w2, torch.bfloat16)
    dgu = torch.empty(M, 2 * fp, dtype=torch.bfloat16, device="cuda")
    args = (B.GEMM_NT, B.EPI_DSWIGLU, M, fp, K, dzd.data_ptr(), K, w2d.data_ptr(), K, dgu.data_ptr(), 2 * fp, None, gu.data_ptr(), 2 * fp, None, 0, None)
    B.check(B.lib.oases_op_gemm_forced(variant, *args) if variant else B.lib.oases_op_gemm(*args))
    dF = dz.double() @ w2.double().t()
    gs = gu.float().cpu().double().reshape(M, fp // 32, 2, 32)
    gst, ust = gs[:, :, 0].reshape(M, fp), gs[:, :, 1].reshape(M, fp)   # the stored (rounded) pre-activations are what backward reads
    ref = interleave(dF * ust * ll.silu_grad(gst), dF * ll.silu(gst))
    assert_bf16_close(dgu.float(), ref, 1e-4, 1e-5)


@pytest.mark.parametrize("variant,M,fp,K", [(201128256, 256, 512, 192), (201128256, 384, 256, 1088), (201256256, 512, 256, 160), (301128256, 256, 512, 192),
                                              (301128256, 392, 288, 1088), (301256256, 512, 256, 160), (0, 4096, 1536, 4096)])
def test_gemm_swiglu_gradient_on_direct_to_lds_kernels(B, ll, variant, M, fp, K):
    """The SwiGLU-gradient epilogue on the kernels whose tiles arrive by direct-to-LDS loads (forced, and as the library's own
    choice for a shape with whole 128 x 256 tiles); the four-wave 128 x 256 kernel has no forward SwiGLU epilogue and refuses it."""
    g = gen(11)
    dz = bf16_round(randn(g, M, K))
    w2 = bf16_round(randn(g, fp, K, scale=0.05))
    gu_ref = bf16_round(randn(g, M, 2 * fp))
    dzd, w2d, gu = dev(dz, torch.bfloat16), dev(w2, torch.bfloat16), dev(gu_ref, torch.bfloat16)
    dgu = torch.empty(M, 2 * fp, dtype=torch.bfloat16, device="cuda")
    args = (B.GEMM_NT, B.EPI_DSWIGLU, M, fp, K, dzd.data_ptr(), K, w2d.data_ptr(), K, dgu.data_ptr(), 2 * fp, None, gu.data_ptr(), 2 * fp, None, 0, None)
    if variant:
        B.check(B.lib.oases_op_gemm_forced(variant, *args))
    else:
        assert B.lib.oases_op_gemm_variant(B.GEMM_NT, B.EPI_DSWIGLU, M, fp, K, 0) == 301128256
        B.check(B.lib.oases_op_gemm(*args))
    dF = dz.double() @ w2.double().t()
    gs = gu_ref.double().reshape(M, fp // 32, 2, 32)
    gst, ust = gs[:, :, 0].reshape(M, fp), gs[:, :, 1].reshape(M, fp)
    assert_bf16_close(dgu.float(), interleave(dF * ust * ll.silu_grad(gst), dF * ll.silu(gst)), 1e-4, 1e-5)
    if variant == 201128256:     # the four-wave 128 x 256 kernel has no forward SwiGLU epilogue
        f = torch.empty(M, fp // 2, dtype=torch.bfloat16, device="cuda")
        a = torch.zeros(M, K, dtype=torch.bfloat16, device="cuda")
        w = torch.zeros(K, fp, dtype=torch.bfloat16, device="cuda")
        assert B.lib.oases_op_gemm_forced(variant, B.GEMM_NN, B.EPI_SWIGLU, M, fp, K, a.data_ptr(), K, w.data_ptr(), fp, f.data_ptr(), fp // 2, None,
                                          gu.data_ptr(), 2 * fp, None, 0, None) == B.EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("variant,M,fp,K", [(201256256, 256, 128, 32), (201256256, 512, 352, 160), (201256256, 256, 1376, 1056), (301256256, 512, 352, 160),
                                              (301256256, 256, 1376, 1056), (301128256, 264, 352, 192), (301128256, 128, 1376, 1088), (0, 4096, 1376, 512)])
def test_gemm_swiglu_forward_on_direct_to_lds_kernel(B, ll, variant, M, fp, K):
    """The SwiGLU epilogue on the kernels whose tiles arrive by direct-to-LDS loads (256 x 256 with four or eight waves, 128 x 256
    with eight): whole and ragged column tiles
    (the interleaved [gate 32 | up 32] blocks end inside the last tile), forced and as the library's choice for LLaMA-7B's
    FC1 width per rank."""
    g = gen(13)
    a = bf16_round(randn(g, M, K))
    wg, wu = bf16_round(randn(g, K, fp, scale=0.05)), bf16_round(randn(g, K, fp, scale=0.05))
    ad, wd = dev(a, torch.bfloat16), dev(interleave(wg, wu), torch.bfloat16)
    f = torch.full((M, fp + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    gu = torch.full((M, 2 * fp + 8), 7.0, dtype=torch.bfloat16, device="cuda")
    args = (B.GEMM_NN, B.EPI_SWIGLU, M, 2 * fp, K, ad.data_ptr(), K, wd.data_ptr(), 2 * fp, f.data_ptr(), fp + 8, None, gu.data_ptr(), 2 * fp + 8, None, 0, None)
    if variant:
        B.check(B.lib.oases_op_gemm_forced(variant, *args))
    else:
        assert B.lib.oases_op_gemm_variant(B.GEMM_NN, B.EPI_SWIGLU, M, 2 * fp, K, 0) == 301256256
        B.check(B.lib.oases_op_gemm(*args))
    gate, up = a.double() @ wg.double(), a.double() @ wu.double()
    assert_bf16_close(gu[:, :2 * fp].float(), interleave(gate, up), 1e-5, 2e-6 * float(gate.abs().max()))
    assert_bf16_close(f[:, :fp].float(), ll.silu(gate) * up, 1e-4, 1e-5)
    assert bool((f[:, fp:] == 7.0).all()) and bool((gu[:, 2 * fp:] == 7.0).all())


def test_gemm_swiglu_argument_errors(B):
    a = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64, 128, dtype=torch.bfloat16, device="cuda")
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    call = lambda op, epi, N, aux, ldaux, ldc: B.lib.oases_op_gemm(op, epi, 64, N, 64, a.data_ptr(), 64, a.data_ptr(), 64, c.data_ptr(), ldc, None,
                                                                   aux, ldaux, None, 0, None)
    assert call(B.GEMM_NT, B.EPI_SWIGLU, 64, c.data_ptr(), 64, 32) == B.EINVAL      # forward epilogue on the NT form
    assert call(B.GEMM_NN, B.EPI_SWIGLU, 32, c.data_ptr(), 32, 16) == B.EINVAL      # N not a multiple of 64
    assert call(B.GEMM_NN, B.EPI_DSWIGLU, 32, c.data_ptr(), 64, 64) == B.EINVAL     # gradient epilogue on the NN form
    assert call(B.GEMM_NT, B.EPI_DSWIGLU, 32, c.data_ptr(), 32, 64) == B.EINVAL     # aux narrower than 2N
    # k slices are never used with these epilogues, even when asked for
    assert B.lib.oases_op_gemm_forced(2128128, B.GEMM_NN, B.EPI_SWIGLU, 64, 64, 64, a.data_ptr(), 64, a.data_ptr(), 64, c.data_ptr(), 32, None,
                                      c.data_ptr(), 64, ws.data_ptr(), ws.numel(), None) == B.EINVAL
    torch.cuda.synchronize()
