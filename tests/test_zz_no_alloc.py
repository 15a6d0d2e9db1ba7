"""The allocation-free column sum (oases_op_colsum_bf16_static) against the scratch-buffer entry point it is a variant
of: two calls in a row on one GPU, the second on a smaller input (the static array keeps the first call's contents),
then the size limit.  Collected last on purpose: a failure here must not hide the parity tests."""
import pytest
import torch

from tests.util import rel_err, bf16_round, dev, randn

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2305_16121_amd import binding
    return binding


def _both(B, rows, cols, ld, seed):
    g = torch.Generator()
    g.manual_seed(seed)
    a = dev(bf16_round(randn(g, rows, ld)), torch.bfloat16)
    ref = torch.full((cols,), 2.0, dtype=torch.float32, device="cuda")
    out = ref.clone()
    scratch = torch.empty(1024 * cols, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    B.check(B.lib.oases_op_colsum_bf16(a.data_ptr(), ld, rows, cols, ref.data_ptr(), scratch.data_ptr(), None))
    B.check(B.lib.oases_op_colsum_bf16_static(a.data_ptr(), ld, rows, cols, out.data_ptr(), None))
    torch.cuda.synchronize()
    return out.cpu(), ref.cpu(), 2.0 + a.cpu().double()[:, :cols].sum(0)


def test_static_colsum_matches_scratch_entry_point_twice_second_smaller(B):
    for (rows, cols, ld, seed) in [(4104, 4096, 4104, 11), (37, 520, 528, 12), (9000, 1536, 1536, 13)]:
        out, ref, exact = _both(B, rows, cols, ld, seed)
        assert torch.equal(out, ref), f"rows={rows} cols={cols}: static and scratch-buffer results differ"   # same kernels: bit for bit
        assert rel_err(out, exact) < 1e-5


def test_static_colsum_rejects_oversized(B):
    a = torch.zeros(8, 4104, dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(4104, dtype=torch.float32, device="cuda")
    rc = B.lib.oases_op_colsum_bf16_static(a.data_ptr(), 4104, 8, 4104, out.data_ptr(), None)
    assert rc == B.EWORKSPACE and b"4096" in B.lib.oases_last_error()
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
