"""Per-operator parity of the HIP kernels (through the C ABI) against the oracle's operator
definitions, on seeded inputs that span several tiles and a ragged tail."""
import math

import numpy as np
import pytest
import torch

from tests.util import rel_err, rms_err, bf16_round, bf16_close, assert_bf16_close, dev, randn

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


def gen(seed):
    g = torch.Generator()
    g.manual_seed(seed)
    return g


# ------------------------------------------------------------------ dropout mask: bit exact
@pytest.mark.parametrize("p,row0,rows,h", [(0.1, 0, 64, 512), (0.5, 1000, 37, 264), (0.1, (1 << 31) // 512, 16, 512), (0.0, 0, 8, 64)])
def test_dropout_mask_bits(B, lo, p, row0, rows, h):
    seed = 0x0123456789ABCDEF
    m = torch.empty(rows * h, dtype=torch.uint8, device="cuda")
    B.check(B.lib.oases_op_dropout_mask(m.data_ptr(), seed, 3, 1, row0, rows, h, p, None))
    torch.cuda.synchronize()
    ref = lo.dropout_keep_mask(seed, 3, 1, rows, h, p, row0=row0)
    assert np.array_equal(m.cpu().numpy().reshape(rows, h).astype(bool), ref)


# ------------------------------------------------------------------ LayerNorm forward
@pytest.mark.parametrize("rows,h", [(300, 512), (70, 1000), (33, 4096), (9, 8192), (5, 16384), (4, 8)])
def test_layernorm_fwd(B, lo, rows, h):
    g = gen(1)
    x = randn(g, rows, h) * 3 + 0.5
    gam, bet = 1 + 0.1 * randn(g, h), 0.1 * randn(g, h)
    xd, gd, bd = dev(x, torch.float32), dev(gam, torch.float32), dev(bet, torch.float32)
    out = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    mu = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mu)
    B.check(B.lib.oases_op_layernorm_fwd(xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), out.data_ptr(), mu.data_ptr(),
                                         rstd.data_ptr(), rows, h, 1e-5, None))
    ref, rmu, rrstd = lo.layer_norm_fwd(xd.cpu().double(), gd.cpu().double(), bd.cpu().double(), 1e-5)
    assert_bf16_close(out.float(), ref, 1e-5, 2e-6 * float(ref.abs().max()))
    assert rel_err(mu, rmu.flatten()) < 1e-5 and rel_err(rstd, rrstd.flatten()) < 1e-5


def test_layernorm_fwd_large_mean(B, lo):
    """Rows whose mean is far from zero compared with their spread: the one-pass statistics must not cancel."""
    g = gen(12)
    rows, h = 64, 4096
    x = randn(g, rows, h) * 0.5 + 300.0 * randn(g, rows, 1)
    xd = dev(x, torch.float32)
    gd, bd = dev(torch.ones(h), torch.float32), dev(torch.zeros(h), torch.float32)
    out = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    mu = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mu)
    B.check(B.lib.oases_op_layernorm_fwd(xd.data_ptr(), gd.data_ptr(), bd.data_ptr(), out.data_ptr(), mu.data_ptr(),
                                         rstd.data_ptr(), rows, h, 1e-5, None))
    ref, rmu, rrstd = lo.layer_norm_fwd(xd.cpu().double(), gd.cpu().double(), bd.cpu().double(), 1e-5)
    assert rel_err(mu, rmu.flatten()) < 1e-6 and rel_err(rstd, rrstd.flatten()) < 1e-3
    assert rel_err(out.float(), ref) < 2e-2      # x itself carries only 2^-24 * 300 of absolute precision in fp32


# ------------------------------------------------------------------ reduction point + bias + dropout + residual (+LN)
@pytest.mark.parametrize("rows,h,p,with_peer,with_ln", [(130, 512, 0.1, True, True), (40, 2048, 0.0, False, True),
                                                        (17, 8192, 0.3, True, False), (64, 1032, 0.1, False, True)])
def test_bias_dropout_residual_ln(B, lo, rows, h, p, with_peer, with_ln):
    g = gen(2)
    part, peer, xin = randn(g, rows, h), randn(g, rows, h), randn(g, rows, h)
    bias, gam, bet = 0.1 * randn(g, h), 1 + 0.1 * randn(g, h), 0.1 * randn(g, h)
    d = {k: dev(v, torch.float32) for k, v in dict(part=part, peer=peer, xin=xin, bias=bias, gam=gam, bet=bet).items()}
    xo = torch.empty(rows, h, dtype=torch.float32, device="cuda")
    ln = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    mu = torch.empty(rows, dtype=torch.float32, device="cuda")
    rstd = torch.empty_like(mu)
    seed, layer, site, row0 = 77, 2, 0, 4096
    B.check(B.lib.oases_op_bias_dropout_residual_ln(
        d["part"].data_ptr(), d["peer"].data_ptr() if with_peer else None, d["bias"].data_ptr(), d["xin"].data_ptr(),
        xo.data_ptr(), d["gam"].data_ptr() if with_ln else None, d["bet"].data_ptr() if with_ln else None,
        ln.data_ptr() if with_ln else None, mu.data_ptr() if with_ln else None, rstd.data_ptr() if with_ln else None,
        rows, h, 1e-5, seed, layer, site, row0, p, None))
    keep = torch.from_numpy(lo.dropout_keep_mask(seed, layer, site, rows, h, p, row0=row0)).double()
    c = {k: v.cpu().double() for k, v in d.items()}
    z = c["part"] + (c["peer"] if with_peer else 0) + c["bias"]
    ref = c["xin"] + keep * z / (1 - p)
    assert rel_err(xo, ref) < 1e-6
    if with_ln:
        rln, rmu, rrstd = lo.layer_norm_fwd(ref, c["gam"], c["bet"], 1e-5)
        assert_bf16_close(ln.float(), rln, 1e-5, 2e-6 * float(rln.abs().max()))
        assert rel_err(mu, rmu.flatten()) < 1e-5 and rel_err(rstd, rrstd.flatten()) < 1e-5


# ------------------------------------------------------------------ dropout backward + bias gradient
@pytest.mark.parametrize("rows,h,p", [(300, 512, 0.1), (1000, 1032, 0.5), (7, 8192, 0.0)])
def test_dropout_bwd(B, lo, rows, h, p):
    g = gen(3)
    dy = dev(randn(g, rows, h), torch.float32)
    dz = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    db = torch.full((h,), 1.0, dtype=torch.float32, device="cuda")      # accumulated into
    scratch = torch.empty(1024 * h, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_dropout_bwd(dy.data_ptr(), dz.data_ptr(), db.data_ptr(), rows, h, 5, 1, 1, 64, p, scratch.data_ptr(), None))
    keep = torch.from_numpy(lo.dropout_keep_mask(5, 1, 1, rows, h, p, row0=64)).double()
    ref = keep * dy.cpu().double() / (1 - p)
    assert_bf16_close(dz.float(), ref, 1e-6)
    assert rel_err(db, 1.0 + ref.sum(0)) < 1e-5


# ------------------------------------------------------------------ LayerNorm backward fusion
@pytest.mark.parametrize("rows,h,p,with_peer,with_dz", [(300, 512, 0.1, True, True), (1000, 1032, 0.0, False, False),
                                                        (50, 8192, 0.2, True, True), (520, 4096, 0.1, False, True)])
def test_layernorm_bwd(B, lo, rows, h, p, with_peer, with_dz):
    g = gen(4)
    part, peer, dres, x = randn(g, rows, h), randn(g, rows, h), randn(g, rows, h), randn(g, rows, h) * 2 + 1
    gam = 1 + 0.1 * randn(g, h)
    d = {k: dev(v, torch.float32) for k, v in dict(part=part, peer=peer, dres=dres, x=x, gam=gam).items()}
    c = {k: v.cpu().double() for k, v in d.items()}
    _, rmu, rrstd = lo.layer_norm_fwd(c["x"], c["gam"], torch.zeros(h, dtype=torch.float64), 1e-5)
    mu, rstd = dev(rmu.flatten(), torch.float32), dev(rrstd.flatten(), torch.float32)
    dxo = torch.empty(rows, h, dtype=torch.float32, device="cuda")
    dz = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    dgam = torch.zeros(h, dtype=torch.float32, device="cuda")
    dbet = torch.zeros_like(dgam)
    dbias = torch.zeros_like(dgam)
    scratch = torch.empty(3 * 1024 * h, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_layernorm_bwd(
        d["part"].data_ptr(), d["peer"].data_ptr() if with_peer else None, d["dres"].data_ptr(), d["x"].data_ptr(),
        mu.data_ptr(), rstd.data_ptr(), d["gam"].data_ptr(), dxo.data_ptr(), dgam.data_ptr(), dbet.data_ptr(),
        dz.data_ptr() if with_dz else None, dbias.data_ptr() if with_dz else None, rows, h, 9, 0, 1, 128, p,
        scratch.data_ptr(), None))
    gin = c["part"] + (c["peer"] if with_peer else 0)
    rdx, rdg, rdb = lo.layer_norm_bwd(gin, c["x"], mu.cpu().double()[:, None], rstd.cpu().double()[:, None], c["gam"])
    ref = c["dres"] + rdx
    assert rel_err(dxo, ref) < 2e-5
    assert rel_err(dgam, rdg) < 2e-5 and rel_err(dbet, rdb) < 2e-5
    if with_dz:
        keep = torch.from_numpy(lo.dropout_keep_mask(9, 0, 1, rows, h, p, row0=128)).double()
        rz = keep * ref / (1 - p)
        assert_bf16_close(dz.float(), rz, 1e-5, 2e-6 * float(rz.abs().max()))
        assert rel_err(dbias, rz.sum(0)) < 2e-5


# ------------------------------------------------------------------ column sums
@pytest.mark.parametrize("rows,cols,ld", [(1000, 768, 768), (37, 4096, 4104), (300, 8, 16)])
def test_colsum(B, rows, cols, ld):
    a = dev(bf16_round(randn(gen(5), rows, ld)), torch.bfloat16)
    out = torch.full((cols,), 2.0, dtype=torch.float32, device="cuda")
    scratch = torch.empty(1024 * cols, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_colsum_bf16(a.data_ptr(), ld, rows, cols, out.data_ptr(), scratch.data_ptr(), None))
    assert rel_err(out, 2.0 + a.cpu().double()[:, :cols].sum(0)) < 1e-5


# ------------------------------------------------------------------ GEMM family
GEMM_SHAPES = [(256, 256, 256), (384, 768, 512), (136, 264, 72), (2048, 1024, 1024), (8, 8, 8), (520, 128, 4096), (4096, 4096, 512)]


@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
@pytest.mark.parametrize("op", ["NN", "NT", "TN"])
def test_gemm_plain(B, M, N, K, op):
    g = gen(6)
    a = bf16_round(randn(g, M, K))
    b = bf16_round(randn(g, K, N))
    ref = a @ b
    if op == "NN":
        ad, bd = dev(a, torch.bfloat16), dev(b, torch.bfloat16)
        c = torch.empty(M, N, dtype=torch.float32, device="cuda")
        B.check(B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_F32, M, N, K, ad.data_ptr(), K, bd.data_ptr(), N, c.data_ptr(), N, None, None, 0, None, 0, None))
    elif op == "NT":
        ad, bd = dev(a, torch.bfloat16), dev(b.t().contiguous(), torch.bfloat16)
        c = torch.empty(M, N, dtype=torch.float32, device="cuda")
        B.check(B.lib.oases_op_gemm(B.GEMM_NT, B.EPI_F32, M, N, K, ad.data_ptr(), K, bd.data_ptr(), K, c.data_ptr(), N, None, None, 0, None, 0, None))
    else:
        ad, bd = dev(a.t().contiguous(), torch.bfloat16), dev(b, torch.bfloat16)
        c = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")         # accumulated into
        B.check(B.lib.oases_op_gemm(B.GEMM_TN, 0, M, N, K, ad.data_ptr(), M, bd.data_ptr(), N, c.data_ptr(), N, None, None, 0, None, 0, None))
        ref = ref + 0.5
    assert rel_err(c, ref) < 1e-5, (op, M, N, K)     # exact products of bf16 values, fp32 accumulation


GEMM_VARIANTS = [1256256, 1128256, 1256128, 101128256, 101256128, 1128128, 2256256, 102128256, 102256128, 3128128]


@pytest.mark.parametrize("variant", GEMM_VARIANTS)
@pytest.mark.parametrize("op", ["NN", "NT", "TN"])
def test_gemm_every_variant(B, lo, op, variant):
    """Every compiled instantiation (block tile, wave grid, k slices), named explicitly, on a shape with several tiles
    in both directions, ragged edges and a ragged k tail; plus the bias+GeLU / dGeLU epilogues of the same variant."""
    M, N, K = 776, 1032, 712
    g = gen(variant % 1000 + variant // 1000000)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    ref = a @ b
    ws = torch.full((32 << 20,), 0xFF, dtype=torch.uint8, device="cuda")
    opc = {"NN": B.GEMM_NN, "NT": B.GEMM_NT, "TN": B.GEMM_TN}[op]
    ad = dev(a if op != "TN" else a.t().contiguous(), torch.bfloat16)
    bd = dev(b if op != "NT" else b.t().contiguous(), torch.bfloat16)
    lda, ldb = (K if op != "TN" else M), (N if op != "NT" else K)
    c = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, None, 0,
                                       ws.data_ptr(), ws.numel(), None))
    assert rel_err(c, ref + (0.5 if op == "TN" else 0.0)) < 1e-5, (op, variant)
    if op == "TN":
        return
    bias = dev(0.1 * randn(g, N), torch.float32)
    pre = dev(bf16_round(randn(g, M, N)), torch.bfloat16)
    cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    if op == "NN":
        aux = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BIAS_GELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           bias.data_ptr(), aux.data_ptr(), N, ws.data_ptr(), ws.numel(), None))
        z = ref + bias.cpu().double()
        assert_bf16_close(aux.float(), z, 1e-5, 2e-6 * float(z.abs().max()))
        assert_bf16_close(cb.float(), lo.gelu_fwd(z), 1e-4, 1e-5)
    else:
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_DGELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           None, pre.data_ptr(), N, ws.data_ptr(), ws.numel(), None))
        assert_bf16_close(cb.float(), ref * lo.gelu_grad(pre.float().cpu().double()), 1e-4, 1e-5)


@pytest.mark.parametrize("M,N,K", [(256, 256, 32), (512, 768, 96), (768, 256, 4096), (1024, 1024, 1056)])
@pytest.mark.parametrize("op", ["NN", "NT", "TN"])
@pytest.mark.parametrize("variant", [201256256, 301256256])
def test_gemm_direct_to_lds_variant(B, lo, op, M, N, K, variant):
    """The kernel whose tiles arrive by direct-to-LDS loads (variant 2xxxxxxxx: whole 256 x 256 tiles, K % 32 == 0): one to
    33 k tiles (prologue-only, tail and steady-state paths of its four-stage pipeline), every contraction form, and the
    epilogues it supports.  301256256: the eight-wave kernel on the same tiles."""
    g = gen(M + N + K)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    ref = a @ b
    opc = {"NN": B.GEMM_NN, "NT": B.GEMM_NT, "TN": B.GEMM_TN}[op]
    ad = dev(a if op != "TN" else a.t().contiguous(), torch.bfloat16)
    bd = dev(b if op != "NT" else b.t().contiguous(), torch.bfloat16)
    lda, ldb = (K if op != "TN" else M), (N if op != "NT" else K)
    c = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, None, 0,
                                       None, 0, None))
    assert rel_err(c, ref + (0.5 if op == "TN" else 0.0)) < 1e-5, (op, M, N, K)
    if op == "TN":
        return
    bias = dev(0.1 * randn(g, N), torch.float32)
    pre = dev(bf16_round(randn(g, M, N)), torch.bfloat16)
    cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    if op == "NN":
        aux = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BIAS_GELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           bias.data_ptr(), aux.data_ptr(), N, None, 0, None))
        z = ref + bias.cpu().double()
        assert_bf16_close(aux.float(), z, 1e-5, 2e-6 * float(z.abs().max()))
        assert_bf16_close(cb.float(), lo.gelu_fwd(z), 1e-4, 1e-5)
    else:
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_DGELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           None, pre.data_ptr(), N, None, 0, None))
        assert_bf16_close(cb.float(), ref * lo.gelu_grad(pre.float().cpu().double()), 1e-4, 1e-5)
    # shapes it does not cover are refused on the host
    assert B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M - 8, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, None, 0,
                                      None, 0, None) == B.EINVAL


@pytest.mark.parametrize("variant,M,N,K", [(v, *mnk) for v in (201128256, 301128256) for mnk in
                                           [(128, 256, 64), (384, 512, 128), (256, 768, 192), (640, 256, 4096), (1152, 1024, 1088), (128, 512, 320)]])
@pytest.mark.parametrize("op", ["NN", "NT", "TN"])
def test_gemm_direct_to_lds_rect_variant(B, lo, op, variant, M, N, K):
    """The kernel with 128 x 256 tiles fed by direct-to-LDS loads (variant 201128256; K % 64 == 0), here on whole tiles: one to 64
    k tiles (prologue-only, drain and steady-state paths of its three-stage pipeline), odd and even tile counts, every
    contraction form, a padded leading dimension of C, and the epilogues it supports."""
    g = gen(M + N + K)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    ref = a @ b
    opc = {"NN": B.GEMM_NN, "NT": B.GEMM_NT, "TN": B.GEMM_TN}[op]
    ad = dev(a if op != "TN" else a.t().contiguous(), torch.bfloat16)
    bd = dev(b if op != "NT" else b.t().contiguous(), torch.bfloat16)
    lda, ldb = (K if op != "TN" else M), (N if op != "NT" else K)
    ldc = N + 64
    c0 = randn(g, M, ldc).float()
    c = dev(c0, torch.float32)
    B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), ldc, None, None, 0,
                                       None, 0, None))
    out = c.cpu().double()
    assert rel_err(out[:, :N], ref + (c0[:, :N].double() if op == "TN" else 0.0)) < 1e-5, (op, M, N, K)   # TN accumulates into C
    assert torch.equal(out[:, N:], c0[:, N:].double())  # the padding columns of C are not touched
    # shapes it does not cover are refused on the host
    assert B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K - 32, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), ldc, None, None, 0,
                                      None, 0, None) == B.EINVAL
    if op == "TN":
        return
    bias = dev(0.1 * randn(g, N), torch.float32)
    pre = dev(bf16_round(randn(g, M, N)), torch.bfloat16)
    cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BF16, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N, None, None, 0,
                                       None, 0, None))
    assert_bf16_close(cb.float(), ref, 1e-5, 2e-6 * float(ref.abs().max()))
    if op == "NN":
        aux = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BIAS_BF16, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           bias.data_ptr(), None, 0, None, 0, None))
        z = ref + bias.cpu().double()
        assert_bf16_close(cb.float(), z, 1e-5, 2e-6 * float(z.abs().max()))
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BIAS_GELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           bias.data_ptr(), aux.data_ptr(), N, None, 0, None))
        assert_bf16_close(aux.float(), z, 1e-5, 2e-6 * float(z.abs().max()))
        assert_bf16_close(cb.float(), lo.gelu_fwd(z), 1e-4, 1e-5)
    else:
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_DGELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                           None, pre.data_ptr(), N, None, 0, None))
        assert_bf16_close(cb.float(), ref * lo.gelu_grad(pre.float().cpu().double()), 1e-4, 1e-5)


@pytest.mark.parametrize("variant,op,M,N,K", [(201128256, "TN", 136, 264, 64), (201128256, "TN", 1376, 1000, 192), (201128256, "TN", 88, 8, 128),
                                              (201128256, "NN", 256, 264, 128), (201128256, "NN", 392, 1000, 1088), (201128256, "NN", 8, 8, 64),
                                              (201128256, "NT", 136, 264, 64), (201128256, "NT", 1000, 1376, 320), (201128256, "NT", 72, 40, 128),
                                              (0, "NT", 4096, 1376, 4096), (201256256, "TN", 264, 520, 96),
                                              (201256256, "TN", 1000, 1376, 160), (201256256, "TN", 8, 8, 32), (201256256, "NN", 512, 776, 224),
                                              (0, "TN", 1376, 4096, 2048), (0, "TN", 4096, 2752, 1024),
                                              (301128256, "TN", 136, 264, 64), (301128256, "TN", 1376, 1000, 192), (301128256, "TN", 88, 8, 128),
                                              (301128256, "NN", 256, 264, 128), (301128256, "NN", 392, 1000, 1088), (301128256, "NN", 8, 8, 64),
                                              (301128256, "NT", 136, 264, 64), (301128256, "NT", 1000, 1376, 320), (301128256, "NT", 72, 40, 128),
                                              (301256256, "TN", 264, 520, 96), (301256256, "TN", 1000, 1376, 160), (301256256, "TN", 8, 8, 32),
                                              (301256256, "NN", 512, 776, 224)])
def test_gemm_direct_to_lds_ragged_edges(B, lo, variant, op, M, N, K):
    """Operands may end inside the last tile of the direct-to-LDS kernels (128 x 256: any operand; 256 x 256: a row-indexed
    one, i.e. A of the TN form and B of the NN and TN forms): the rows / chunks beyond them are fetched from valid memory
    and what they feed is never stored.  Forced on both kernels, and as the library's own choice for LLaMA-7B's FFN
    weight-gradient and input-gradient shapes.  C sits inside a larger buffer whose other bytes must stay as they were."""
    g = gen(M + N + K)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    ref = a @ b
    opc = {"NN": B.GEMM_NN, "NT": B.GEMM_NT, "TN": B.GEMM_TN}[op]
    ad = dev(a if op != "TN" else a.t().contiguous(), torch.bfloat16)
    bd = dev(b if op != "NT" else b.t().contiguous(), torch.bfloat16)
    lda, ldb = (K if op != "TN" else M), (N if op != "NT" else K)
    ldc = N + 40
    guard = 3                                               # rows of C's buffer before and after the matrix
    c0 = randn(g, M + 2 * guard, ldc).float()
    c = dev(c0, torch.float32)
    cptr = c.data_ptr() + guard * ldc * 4
    if variant:
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cptr, ldc, None, None, 0, None, 0, None))
    else:
        assert B.lib.oases_op_gemm_variant(opc, B.EPI_DGELU if op == "NT" else B.EPI_F32, M, N, K, 0) >= 200000000
        B.check(B.lib.oases_op_gemm(opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cptr, ldc, None, None, 0, None, 0, None))
    out = c.cpu()
    body = out[guard:guard + M].double()
    assert rel_err(body[:, :N], ref + (c0[guard:guard + M, :N].double() if op == "TN" else 0.0)) < 1e-5, (op, M, N, K)
    assert torch.equal(body[:, N:], c0[guard:guard + M, N:].double())
    assert torch.equal(out[:guard], c0[:guard]) and torch.equal(out[guard + M:], c0[guard + M:])
    if op == "NN":                                          # a fused epilogue on a ragged tile
        bias = dev(0.1 * randn(g, N), torch.float32)
        cb = torch.full((M, N + 8), 7.0, dtype=torch.bfloat16, device="cuda")
        aux = torch.full((M, N + 8), 7.0, dtype=torch.bfloat16, device="cuda")
        B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BIAS_GELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), N, cb.data_ptr(), N + 8,
                                           bias.data_ptr(), aux.data_ptr(), N + 8, None, 0, None))
        z = ref + bias.cpu().double()
        assert_bf16_close(aux[:, :N].float(), z, 1e-5, 2e-6 * float(z.abs().max()))
        assert_bf16_close(cb[:, :N].float(), lo.gelu_fwd(z), 1e-4, 1e-5)
        assert bool((cb[:, N:] == 7.0).all()) and bool((aux[:, N:] == 7.0).all())
    if op == "NT":                                          # (for variant 0: the launch the library itself picks for this epilogue)
        pre = dev(bf16_round(randn(g, M, N)), torch.bfloat16)
        cb = torch.full((M, N + 8), 7.0, dtype=torch.bfloat16, device="cuda")
        args = (opc, B.EPI_DGELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N + 8, None, pre.data_ptr(), N, None, 0, None)
        B.check(B.lib.oases_op_gemm_forced(variant, *args) if variant else B.lib.oases_op_gemm(*args))
        assert_bf16_close(cb[:, :N].float(), ref * lo.gelu_grad(pre.float().cpu().double()), 1e-4, 1e-5)
        assert bool((cb[:, N:] == 7.0).all())


@pytest.mark.parametrize("K,M0,N0,M1,N1", [(64, 128, 256, 128, 256), (192, 256, 512, 384, 256), (4096, 128, 768, 640, 256), (1088, 512, 1024, 1152, 768)])
def test_gemm_tn_pair(B, K, M0, N0, M1, N1):
    """Two weight gradients in one launch: each result is the product (accumulated into C, padded leading dimensions
    untouched) and is bit-identical to the same kernel launched for that problem alone."""
    g = gen(K + M0 + N1)
    prob = []
    for (M, N) in ((M0, N0), (M1, N1)):
        a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
        lda, ldb, ldc = M + 8, N + 16, N + 64
        ap, bp = torch.zeros(K, lda, dtype=torch.float64), torch.zeros(K, ldb, dtype=torch.float64)
        ap[:, :M], bp[:, :N] = a.t(), b
        c0 = randn(g, M, ldc).float()
        prob.append(dict(M=M, N=N, ref=a @ b, ad=dev(ap, torch.bfloat16), bd=dev(bp, torch.bfloat16), lda=lda, ldb=ldb, ldc=ldc, c0=c0,
                         c=dev(c0, torch.float32), c_alone=dev(c0, torch.float32)))
    p0, p1 = prob
    B.check(B.lib.oases_op_gemm_tn_pair(K, M0, N0, p0["ad"].data_ptr(), p0["lda"], p0["bd"].data_ptr(), p0["ldb"], p0["c"].data_ptr(), p0["ldc"],
                                        M1, N1, p1["ad"].data_ptr(), p1["lda"], p1["bd"].data_ptr(), p1["ldb"], p1["c"].data_ptr(), p1["ldc"], None))
    for q in prob:
        B.check(B.lib.oases_op_gemm_forced(201128256, B.GEMM_TN, B.EPI_F32, q["M"], q["N"], K, q["ad"].data_ptr(), q["lda"], q["bd"].data_ptr(), q["ldb"],
                                           q["c_alone"].data_ptr(), q["ldc"], None, None, 0, None, 0, None))
        out = q["c"].cpu().double()
        assert rel_err(out[:, :q["N"]], q["ref"] + q["c0"][:, :q["N"]].double()) < 1e-5
        assert torch.equal(out[:, q["N"]:], q["c0"][:, q["N"]:].double())
        assert torch.equal(q["c"], q["c_alone"])
    # shapes the kernel does not cover, NULL and misaligned operands: refused on the host
    args = lambda **o: [o.get("K", K), o.get("M0", M0), N0, o.get("A0", p0["ad"].data_ptr()), p0["lda"], p0["bd"].data_ptr(), p0["ldb"], p0["c"].data_ptr(),
                        p0["ldc"], M1, o.get("N1", N1), p1["ad"].data_ptr(), p1["lda"], p1["bd"].data_ptr(), p1["ldb"], p1["c"].data_ptr(), o.get("ldc1", p1["ldc"]), None]
    assert B.lib.oases_op_gemm_tn_pair(*args(K=K + 32)) == B.EINVAL
    assert B.lib.oases_op_gemm_tn_pair(*args(M0=M0 - 64)) == B.EINVAL
    assert B.lib.oases_op_gemm_tn_pair(*args(N1=N1 - 128)) == B.EINVAL
    assert B.lib.oases_op_gemm_tn_pair(*args(ldc1=N1 - 4)) == B.EINVAL
    assert B.lib.oases_op_gemm_tn_pair(*args(A0=None)) == B.ENULL
    assert B.lib.oases_op_gemm_tn_pair(*args(A0=p0["ad"].data_ptr() + 2)) == B.EALIGN
    torch.cuda.synchronize()


@pytest.mark.parametrize("variant,op,M,N,K", [(202128256, "NN", 256, 512, 256), (202128256, "NT", 136, 264, 384), (204128256, "NN", 128, 256, 1024),
                                              (202128256, "TN", 392, 1000, 640), (204128256, "NT", 1024, 512, 4096),
                                              (302128256, "NN", 256, 512, 256), (302128256, "NT", 136, 264, 384), (304128256, "NN", 128, 256, 1024),
                                              (302128256, "TN", 392, 1000, 640), (304128256, "NT", 1024, 512, 4096)])
def test_gemm_direct_to_lds_k_slices(B, lo, variant, op, M, N, K):
    """The 128 x 256 direct-to-LDS kernel over two or four k slices of whole stages (variants 202128256, 204128256): fp32
    partial planes in the workspace, summed in slice order by the second pass, which applies the epilogue."""
    g = gen(M + N + K)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    ref = a @ b
    opc = {"NN": B.GEMM_NN, "NT": B.GEMM_NT, "TN": B.GEMM_TN}[op]
    ad = dev(a if op != "TN" else a.t().contiguous(), torch.bfloat16)
    bd = dev(b if op != "NT" else b.t().contiguous(), torch.bfloat16)
    lda, ldb = (K if op != "TN" else M), (N if op != "NT" else K)
    S = variant // 1000000 % 100
    ws = torch.empty(S * M * N * 4, dtype=torch.uint8, device="cuda")
    c0 = randn(g, M, N + 8).float()
    c = dev(c0, torch.float32)
    B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N + 8, None, None, 0,
                                       ws.data_ptr(), ws.numel(), None))
    out = c.cpu().double()
    assert rel_err(out[:, :N], ref + (c0[:, :N].double() if op == "TN" else 0.0)) < 1e-5
    assert torch.equal(out[:, N:], c0[:, N:].double())
    if op != "TN":
        bias = dev(0.1 * randn(g, N), torch.float32)
        pre = dev(bf16_round(randn(g, M, N)), torch.bfloat16)
        cb = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
        if op == "NN":
            aux = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
            B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_BIAS_GELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                               bias.data_ptr(), aux.data_ptr(), N, ws.data_ptr(), ws.numel(), None))
            z = ref + bias.cpu().double()
            assert_bf16_close(aux.float(), z, 1e-5, 2e-6 * float(z.abs().max()))
            assert_bf16_close(cb.float(), lo.gelu_fwd(z), 1e-4, 1e-5)
        else:
            B.check(B.lib.oases_op_gemm_forced(variant, opc, B.EPI_DGELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, cb.data_ptr(), N,
                                               None, pre.data_ptr(), N, ws.data_ptr(), ws.numel(), None))
            assert_bf16_close(cb.float(), ref * lo.gelu_grad(pre.float().cpu().double()), 1e-4, 1e-5)
    # slices that are not whole stages, or a workspace that is too small: refused on the host
    assert B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K - 64, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N + 8, None, None, 0,
                                      ws.data_ptr(), ws.numel(), None) == B.EINVAL
    assert B.lib.oases_op_gemm_forced(variant, opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N + 8, None, None, 0,
                                      ws.data_ptr(), ws.numel() - 4, None) == B.EINVAL
    torch.cuda.synchronize()


def test_gemm_forced_variant_errors(B):
    """Variants that do not exist, k slices that do not fit K or the workspace: EINVAL before any launch."""
    M = N = K = 256
    a = torch.zeros(M, K, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(M, N, dtype=torch.float32, device="cuda")
    ws = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    call = lambda v, wsb: B.lib.oases_op_gemm_forced(v, B.GEMM_NN, B.EPI_F32, M, N, K, a.data_ptr(), K, a.data_ptr(), N, c.data_ptr(), N, None, None, 0,
                                                     ws.data_ptr(), wsb, None)
    assert call(1128128, ws.numel()) == 0
    for bad in (0, -5, 1192192, 1064064, 101256256, 101128128, 201256128, 201128128, 301128128, 401128256, 308128256, 9128128, 128128):
        assert call(bad, ws.numel()) == B.EINVAL, bad
    assert call(2128128, 1024) == B.EINVAL           # workspace too small for two planes
    assert call(8128128, ws.numel()) == B.EINVAL     # 8 slices of 64 do not all start inside K = 256
    torch.cuda.synchronize()


def test_gemm_operand_that_spans_2gib_takes_the_staged_kernel(B):
    """The direct-to-LDS kernels address an operand with 32-bit byte offsets.  An A whose rows lie 2^18 elements apart
    spans 2 GiB: the library's own choice still gives the product (register-staged kernel of the same tile), a forced
    direct-to-LDS variant is refused."""
    M, N, K, lda = 4096, 2048, 256, 1 << 18
    g = gen(23)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    big = torch.zeros(M, lda, dtype=torch.bfloat16, device="cuda")
    big[:, :K] = dev(a, torch.bfloat16)
    bd = dev(b, torch.bfloat16)
    c = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
    args = (B.GEMM_NN, B.EPI_F32, M, N, K, big.data_ptr(), lda, bd.data_ptr(), N, c.data_ptr(), N, None, None, 0, None, 0, None)
    assert B.lib.oases_op_gemm_variant(B.GEMM_NN, B.EPI_F32, M, N, K, 0) // 100000000 == 3    # a dense A would go to the eight-wave kernel
    B.check(B.lib.oases_op_gemm(*args))
    torch.cuda.synchronize()
    assert rel_err(c, a.double() @ b.double()) < 1e-5
    for v in (301256256, 201256256, 301128256, 201128256):
        assert B.lib.oases_op_gemm_forced(v, *args) == B.EINVAL, v
    assert "2 GiB" in B.lib.oases_last_error().decode()
    del big
    torch.cuda.empty_cache()


@pytest.mark.parametrize("M,N,K", [(384, 768, 512), (136, 264, 72), (2048, 2048, 256)])
def test_gemm_epilogues(B, lo, M, N, K):
    g = gen(7)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    bias = 0.1 * randn(g, N)
    ad, bd, biasd = dev(a, torch.bfloat16), dev(b, torch.bfloat16), dev(bias, torch.float32)
    bias = biasd.cpu().double()
    acc = a @ b
    c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    aux = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    run = lambda epi, auxp: B.check(B.lib.oases_op_gemm(B.GEMM_NN, epi, M, N, K, ad.data_ptr(), K, bd.data_ptr(), N, c.data_ptr(), N,
                                                        biasd.data_ptr(), auxp, N, None, 0, None))
    run(B.EPI_BF16, None)
    assert_bf16_close(c.float(), acc, 1e-5, 2e-6 * float(acc.abs().max()))
    run(B.EPI_BIAS_BF16, None)
    assert_bf16_close(c.float(), acc + bias, 1e-5, 2e-6 * float(acc.abs().max()))
    run(B.EPI_BIAS_GELU, aux.data_ptr())
    assert_bf16_close(aux.float(), acc + bias, 1e-5, 2e-6 * float(acc.abs().max()))
    assert_bf16_close(c.float(), lo.gelu_fwd(acc + bias), 1e-4, 1e-5, 'gelu')
    # dGeLU epilogue on the input-gradient form: C = (A B^T) * gelu'(aux)
    bt = dev(b.t().contiguous(), torch.bfloat16)
    B.check(B.lib.oases_op_gemm(B.GEMM_NT, B.EPI_DGELU, M, N, K, ad.data_ptr(), K, bt.data_ptr(), K, c.data_ptr(), N, None, aux.data_ptr(), N, None, 0, None))
    assert_bf16_close(c.float(), acc * lo.gelu_grad(aux.cpu().double()), 1e-4, 1e-5, 'dgelu')


@pytest.mark.parametrize("op,epi,M,N,K", [("NT", "bf16", 1024, 1024, 8192), ("TN", "acc", 512, 4096, 8192), ("NN", "bias_gelu", 512, 1024, 8192),
                                          ("NT", "dgelu", 520, 264, 4104), ("NN", "f32", 256, 512, 2048)])
def test_gemm_split_k(B, lo, op, epi, M, N, K):
    """Tile-starved shapes with a workspace: K is split into slices whose fp32 partial planes are added in slice order."""
    g = gen(11)
    a, b = bf16_round(randn(g, M, K)), bf16_round(randn(g, K, N, scale=0.05))
    bias = dev(0.1 * randn(g, N), torch.float32)
    pre = dev(bf16_round(randn(g, M, N)), torch.bfloat16)
    ws = torch.full((64 << 20,), 0xFF, dtype=torch.uint8, device="cuda")
    opc = {"NN": B.GEMM_NN, "NT": B.GEMM_NT, "TN": B.GEMM_TN}[op]
    variant = B.lib.oases_op_gemm_variant(opc, 0, M, N, K, ws.numel())
    assert variant // 1000000 % 100 >= 2, f"shape was expected to split K, got {variant}"
    ad = dev(a if op != "TN" else a.t().contiguous(), torch.bfloat16)
    bd = dev(b if op != "NT" else b.t().contiguous(), torch.bfloat16)
    lda = K if op != "TN" else M
    ldb = N if op != "NT" else K
    acc = a @ b
    res = []
    for wsp, wsb in ((ws.data_ptr(), ws.numel()), (None, 0)):
        if epi == "acc":
            c = torch.full((M, N), 0.25, dtype=torch.float32, device="cuda")
            B.check(B.lib.oases_op_gemm(opc, 0, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, None, 0, wsp, wsb, None))
            assert rel_err(c, acc + 0.25) < 1e-5
        elif epi == "f32":
            c = torch.empty(M, N, dtype=torch.float32, device="cuda")
            B.check(B.lib.oases_op_gemm(opc, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, None, 0, wsp, wsb, None))
            assert rel_err(c, acc) < 1e-5
        elif epi == "bf16":
            c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
            B.check(B.lib.oases_op_gemm(opc, B.EPI_BF16, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, None, 0, wsp, wsb, None))
            assert_bf16_close(c.float(), acc, 1e-5, 2e-6 * float(acc.abs().max()))
        elif epi == "bias_gelu":
            c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
            aux = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
            B.check(B.lib.oases_op_gemm(opc, B.EPI_BIAS_GELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, bias.data_ptr(),
                                        aux.data_ptr(), N, wsp, wsb, None))
            z = acc + bias.cpu().double()
            assert_bf16_close(aux.float(), z, 1e-5, 2e-6 * float(z.abs().max()))
            assert_bf16_close(c.float(), lo.gelu_fwd(z), 1e-4, 1e-5)
        else:
            c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
            B.check(B.lib.oases_op_gemm(opc, B.EPI_DGELU, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), N, None, pre.data_ptr(), N,
                                        wsp, wsb, None))
            assert_bf16_close(c.float(), acc * lo.gelu_grad(pre.float().cpu().double()), 1e-4, 1e-5)
        res.append(c.float().cpu())
    assert rel_err(res[0], res[1]) < 3e-2       # split and unsplit agree up to the accumulation order (and one bf16 ulp)


def test_gemm_strided_views(B):
    # operands that are column blocks of wider matrices (the way the layer calls it on sub-batch rows)
    g = gen(8)
    M, N, K, lda, ldb, ldc = 264, 136, 200, 328, 256, 144
    a, b = bf16_round(randn(g, M, lda)), bf16_round(randn(g, K, ldb))
    ad, bd = dev(a, torch.bfloat16), dev(b, torch.bfloat16)
    c = torch.zeros(M, ldc, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_F32, M, N, K, ad.data_ptr(), lda, bd.data_ptr(), ldb, c.data_ptr(), ldc, None, None, 0, None, 0, None))
    assert rel_err(c[:, :N], a[:, :K] @ b[:, :N]) < 1e-5
    assert float(c[:, N:].abs().max()) == 0.0


def test_gemm_argument_errors(B):
    t = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    assert B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_F32, 60, 64, 64, t.data_ptr(), 64, t.data_ptr(), 64, c.data_ptr(), 64, None, None, 0, None, 0, None) == B.EINVAL
    assert B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_F32, 64, 64, 64, None, 64, t.data_ptr(), 64, c.data_ptr(), 64, None, None, 0, None, 0, None) == B.ENULL
    assert B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_F32, 64, 64, 64, t.data_ptr() + 2, 64, t.data_ptr(), 64, c.data_ptr(), 64, None, None, 0, None, 0, None) == B.EALIGN
    assert B.lib.oases_op_gemm(B.GEMM_NN, B.EPI_BIAS_BF16, 64, 64, 64, t.data_ptr(), 64, t.data_ptr(), 64, c.data_ptr(), 64, None, None, 0, None, 0, None) == B.ENULL
    assert b"bias" in B.lib.oases_last_error()


# ------------------------------------------------------------------ attention
def _attn_ref(lo, qkv, batch, seq, heads, d, causal):
    hp = heads * d
    q, k, v = qkv[:, :hp], qkv[:, hp:2 * hp], qkv[:, 2 * hp:]
    A, P = lo.attention_fwd(q, k, v, batch, seq, heads, d, causal)
    return q, k, v, A, P


ATTN_CASES = [(2, 256, 2, 64, 1), (2, 256, 2, 128, 1), (3, 200, 1, 64, 0), (1, 328, 2, 128, 0), (2, 72, 3, 64, 1), (1, 1, 1, 64, 1),
              (1, 1024, 1, 128, 1), (1, 2048, 1, 128, 1),
              (3, 1024, 3, 64, 1)]    # the last one has more than 256 blocks: the backward runs as two launches, not one


@pytest.mark.parametrize("batch,seq,heads,d,causal", ATTN_CASES)
def test_attention_fwd_bwd(B, lo, batch, seq, heads, d, causal):
    g = gen(9)
    M, hp = batch * seq, heads * d
    qkv = bf16_round(randn(g, M, 3 * hp))
    dout = bf16_round(randn(g, M, hp))
    q, k, v, A, P = _attn_ref(lo, qkv, batch, seq, heads, d, causal)
    qd, dod = dev(qkv, torch.bfloat16), dev(dout, torch.bfloat16)
    out = torch.zeros(M, hp, dtype=torch.bfloat16, device="cuda")
    lse = torch.zeros(batch * heads * seq, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_op_attention_fwd(qd.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, seq, heads, d, causal, 0, M, None))
    # P is rounded to bf16 before P*V (relative 2^-9 per weight), then the output is rounded once
    assert_bf16_close(out.float(), A, 0.0, 2.0 ** -9 * float(v.abs().max()), 'attention forward')
    # log-sum-exp of the scaled scores
    S = (lo._heads(q, batch, seq, heads, d) @ lo._heads(k, batch, seq, heads, d).transpose(2, 3)) / math.sqrt(d)
    if causal:
        i = torch.arange(seq)
        S = S.masked_fill(i[None, :] > i[:, None], float("-inf"))
    assert float((lse.cpu().double().reshape(batch, heads, seq) - torch.logsumexp(S, dim=3)).abs().max()) < 2e-3
    # backward consumes the kernel's own rounded output, as the layer does
    dq, dk, dv = lo.attention_bwd(dout, q, k, v, P, batch, seq, heads, d)
    dqkv = torch.zeros(M, 3 * hp, dtype=torch.bfloat16, device="cuda")
    delta = torch.zeros_like(lse)
    B.check(B.lib.oases_op_attention_bwd(qd.data_ptr(), out.data_ptr(), dod.data_ptr(), lse.data_ptr(), delta.data_ptr(),
                                         dqkv.data_ptr(), batch, seq, heads, d, causal, 0, M, None))
    got = dqkv.float().cpu().double()
    got = dict(dq=got[:, :hp], dk=got[:, hp:2 * hp], dv=got[:, 2 * hp:])
    # (a) against the exact definition, element by element, within the bound that the storage formats give.  The kernel
    #     keeps P and dS in fp32 and rounds them to bf16 (half an ulp: relative 2^-8 at most) only where they enter a matrix product; it takes
    #     delta_i = sum_c dO_ic O_ic from the stored output, each O_ic off by the forward's P rounding and its own bf16
    #     rounding; every result is rounded to bf16 once.  First-order propagation of these roundings:
    #       |err dV_j| <= u (sum_i P_ij |dO_i| + |dV_j|),   u = 2^-8
    #       |err dQ_i| <= (u sum_j |dS_ij| |K_j| + e_i sum_j P_ij |K_j|) / sqrt(d) + u |dQ_i|,   dK alike with Q,
    #       e_i = u sum_c |dO_ic| (|O_ic| + sum_j P_ij |V_jc|)   (error of delta_i)
    #     plus 2 % for second-order terms and 1e-5 of the largest value for the fp32 arithmetic.
    Hh, Uu, u9 = (lambda t: lo._heads(t, batch, seq, heads, d)), (lambda t: lo._unheads(t, batch, seq, heads, d)), 2.0 ** -8
    dPx = Hh(dout) @ Hh(v).transpose(2, 3)
    dSx = P * (dPx - (dPx * P).sum(dim=3, keepdim=True))
    e_delta = u9 * (Hh(dout).abs() * (Hh(A).abs() + P @ Hh(v).abs())).sum(dim=3, keepdim=True)
    bound = dict(dv=u9 * (Uu(P.transpose(2, 3) @ Hh(dout).abs()) + dv.abs()),
                 dq=(u9 * Uu(dSx.abs() @ Hh(k).abs()) + Uu((P * e_delta) @ Hh(k).abs())) / math.sqrt(d) + u9 * dq.abs(),
                 dk=(u9 * Uu(dSx.abs().transpose(2, 3) @ Hh(q).abs()) + Uu((P * e_delta).transpose(2, 3) @ Hh(q).abs())) / math.sqrt(d) + u9 * dk.abs())
    for name, ref in (("dq", dq), ("dk", dk), ("dv", dv)):
        assert rms_err(got[name], ref) < 6e-3, name
        excess = (got[name] - ref).abs() - (1.02 * bound[name] + 1e-5 * float(ref.abs().max()))
        assert float(excess.max()) <= 0.0, f"{name}: {int((excess > 0).sum())} elements beyond the storage-format bound, worst by {float(excess.max()):.3g}"
    # (b) against the same mathematics with the kernel's storage roundings written out: delta from the bf16 output,
    #     P and dS rounded to bf16 where they enter a matrix product; then only the final bf16 rounding remains
    H = lambda t: lo._heads(t, batch, seq, heads, d)
    Og = out.float().cpu().double()
    dl = (H(dout) * H(Og)).sum(dim=3, keepdim=True)
    dP = H(dout) @ H(v).transpose(2, 3)
    dS = P * (dP - dl)
    U = lambda t: lo._unheads(t, batch, seq, heads, d)
    ref_b = dict(dv=U(bf16_round(P).transpose(2, 3) @ H(dout)), dq=U(bf16_round(dS) @ H(k)) / math.sqrt(d),
                 dk=U(bf16_round(dS).transpose(2, 3) @ H(q)) / math.sqrt(d))
    for name in ("dq", "dk", "dv"):
        r = ref_b[name]
        # a bf16 rounding of P / dS that falls the other way (fp32 vs fp64 in front of it) moves one term by 2^-8
        assert_bf16_close(got[name], r, 3e-3, 6e-3 * float(torch.sqrt((r ** 2).mean())), name)


@pytest.mark.parametrize("d", [64, 128])
def test_attention_sequence_chunks(B, lo, d):
    """Sub-batches that are chunks of one sequence: forward chunk by chunk in order, backward in reverse order,
    must give what one call over whole sequences gives (bit for bit: same tiles, same order of accumulation)."""
    g = gen(10)
    batch, seq, heads, nchunk = 2, 512, 2, 4
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
            B.check(B.lib.oases_op_attention_fwd(qd.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, seq, heads, d, 1, r0, rows, None))
        for r0 in reversed(starts):
            B.check(B.lib.oases_op_attention_bwd(qd.data_ptr(), out.data_ptr(), dod.data_ptr(), lse.data_ptr(), delta.data_ptr(),
                                                 dqkv.data_ptr(), batch, seq, heads, d, 1, r0, rows, None))
        torch.cuda.synchronize()
        res.append((out.clone(), lse.clone(), dqkv.clone()))
    for a, b in zip(*res):
        assert torch.equal(a, b)


@pytest.mark.parametrize("d", [64, 128])
def test_attention_chunks_never_touch_rows_outside_their_range(B, lo, d):
    """Chunks whose boundaries are off the 32-row tile grid.  Forward of a chunk must not depend on later rows of qkv
    (not computed yet when the layer runs it), backward of a chunk not on dout / out / delta rows in front of it:
    those rows are filled with NaN here; results must equal the whole-sequence run."""
    g = gen(13)
    batch, seq, heads, chunk = 1, 264, 2, 88
    M, hp = seq, heads * d
    qkv = bf16_round(randn(g, M, 3 * hp))
    dout = bf16_round(randn(g, M, hp))
    qd, dod = dev(qkv, torch.bfloat16), dev(dout, torch.bfloat16)
    nan = float("nan")
    # reference: one call over the whole sequence
    out0 = torch.zeros(M, hp, dtype=torch.bfloat16, device="cuda")
    lse0 = torch.zeros(heads * seq, dtype=torch.float32, device="cuda")
    dq0 = torch.zeros(M, 3 * hp, dtype=torch.bfloat16, device="cuda")
    dl0 = torch.zeros_like(lse0)
    B.check(B.lib.oases_op_attention_fwd(qd.data_ptr(), out0.data_ptr(), lse0.data_ptr(), batch, seq, heads, d, 1, 0, M, None))
    B.check(B.lib.oases_op_attention_bwd(qd.data_ptr(), out0.data_ptr(), dod.data_ptr(), lse0.data_ptr(), dl0.data_ptr(), dq0.data_ptr(),
                                         batch, seq, heads, d, 1, 0, M, None))
    # chunked: forward in order, rows behind the current chunk poisoned
    out = torch.full((M, hp), nan, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((heads * seq,), nan, dtype=torch.float32, device="cuda")
    for r0 in range(0, M, chunk):
        qpart = qd.clone()
        qpart[r0 + chunk:] = nan
        B.check(B.lib.oases_op_attention_fwd(qpart.data_ptr(), out.data_ptr(), lse.data_ptr(), batch, seq, heads, d, 1, r0, chunk, None))
        torch.cuda.synchronize()
    assert torch.equal(out, out0) and torch.equal(lse, lse0)
    # backward in reverse order, dout / delta rows in front of the current chunk poisoned
    dqkv = torch.full((M, 3 * hp), nan, dtype=torch.bfloat16, device="cuda")
    delta = torch.full_like(lse0, nan)
    for r0 in reversed(range(0, M, chunk)):
        dpart = dod.clone()
        dpart[:r0] = nan
        B.check(B.lib.oases_op_attention_bwd(qd.data_ptr(), out.data_ptr(), dpart.data_ptr(), lse.data_ptr(), delta.data_ptr(),
                                             dqkv.data_ptr(), batch, seq, heads, d, 1, r0, chunk, None))
        torch.cuda.synchronize()
    assert not bool(torch.isnan(dqkv.float()).any())
    # same tiles, but the split of a block's reduction range over the waves depends on where the block starts
    assert rel_err(dqkv.float(), dq0.float()) < 2e-2


def test_attention_argument_errors(B):
    t = torch.zeros(256, 3 * 64, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros(256, 64, dtype=torch.bfloat16, device="cuda")
    l = torch.zeros(256, dtype=torch.float32, device="cuda")
    f = B.lib.oases_op_attention_fwd
    assert f(t.data_ptr(), o.data_ptr(), l.data_ptr(), 2, 128, 1, 96, 1, 0, 256, None) == B.EINVAL       # head_dim
    assert f(t.data_ptr(), o.data_ptr(), l.data_ptr(), 2, 128, 1, 64, 1, 64, 128, None) == B.EINVAL      # straddles sequences
    assert f(t.data_ptr(), o.data_ptr(), l.data_ptr(), 2, 128, 1, 64, 0, 0, 64, None) == B.EINVAL        # chunk, non-causal
    assert f(t.data_ptr(), o.data_ptr(), l.data_ptr(), 2, 128, 1, 64, 1, 0, 512, None) == B.EINVAL       # beyond the batch
    assert f(None, o.data_ptr(), l.data_ptr(), 2, 128, 1, 64, 1, 0, 256, None) == B.ENULL


# ------------------------------------------------------------------ measurement helpers
def test_probe_entry_points(B):
    """The two measurement helpers run and refuse bad arguments (what they measure is reported by bench.py)."""
    out = torch.zeros(64 * 256, dtype=torch.float32, device="cuda")
    B.check(B.lib.oases_probe_mfma_rate(1, 10, 64, out.data_ptr(), None))
    assert B.lib.oases_probe_mfma_rate(0, 0, 64, out.data_ptr(), None) == B.EINVAL
    assert B.lib.oases_probe_mfma_rate(0, 10, 64, None, None) == B.ENULL
    src = torch.zeros(16 * 65536, dtype=torch.uint8, device="cuda")
    for waves in (4, 8):
        B.check(B.lib.oases_probe_lds_load_rate(waves, 20, 16, src.data_ptr(), src.numel(), out.data_ptr(), None))
    assert B.lib.oases_probe_lds_load_rate(6, 20, 16, src.data_ptr(), src.numel(), out.data_ptr(), None) == B.EINVAL
    assert B.lib.oases_probe_lds_load_rate(8, 20, 17, src.data_ptr(), src.numel(), out.data_ptr(), None) == B.EINVAL   # src too small
    assert B.lib.oases_probe_lds_load_rate(8, 20, 16, None, src.numel(), out.data_ptr(), None) == B.ENULL
    torch.cuda.synchronize()
    assert bool((src == 0).all())
