"""The entry point that allocates nothing (dapple_colsum_static, partial sums in an array built into the
library's device code) against the entry point it is a variant of (dapple_colsum, partial sums in a buffer the
caller brings): same kernels, same summation order, so the outputs must agree bit for bit.  Two calls in a row,
the second on a smaller input, so that what the first call left in the shared array cannot leak into the second;
sizes beyond the array are refused before anything is enqueued."""
import numpy as np
import pytest

from paper_2007_01045_amd import binding as B
from paper_2007_01045_amd import inputs as I

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")


def _case(dtype, rows, cols, ld, tag):
    bf = dtype == B.DTYPE_BF16
    X = I.normal(77, tag, rows * ld).reshape(rows, ld)
    X = I.round_to_bf16(X) if bf else X.astype(np.float32)
    dX = torch.from_numpy(np.ascontiguousarray(X)).to("cuda", dtype=torch.bfloat16 if bf else torch.float32)
    start = torch.from_numpy(I.normal(78, tag, cols).astype(np.float32)).cuda()   # out is accumulated into
    partial = torch.empty(((rows + 63) // 64) * cols, dtype=torch.float32, device="cuda")
    ref, got = start.clone(), start.clone()
    B.dapple_colsum(dtype, dX.data_ptr(), rows, cols, ld, partial.data_ptr(), ref.data_ptr())
    B.dapple_colsum_static(dtype, dX.data_ptr(), rows, cols, ld, got.data_ptr())
    torch.cuda.synchronize()
    ref, got = ref.cpu().numpy(), got.cpu().numpy()
    assert np.array_equal(ref, got), (tag, float(np.abs(ref - got).max()))
    # and both are the column sum (float64 on the host), so a pair of equally wrong results cannot pass
    exact = X[:, :cols].astype(np.float64).sum(0) + start.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(got - exact) <= 1e-5 * np.linalg.norm(exact)


@pytest.mark.parametrize("dtype", [B.DTYPE_F32, B.DTYPE_BF16])
def test_static_scratch_colsum_matches_workspace_colsum_twice(dtype):
    _case(dtype, 2048, 4096, 4096, f"big{dtype}")      # 32 blocks x 4096 partial sums
    _case(dtype, 203, 1032, 1040, f"small{dtype}")     # smaller, ragged: 4 blocks x 1032, right after
    _case(dtype, 64, 8, 8, f"tiny{dtype}")


def test_static_scratch_colsum_refuses_what_does_not_fit():
    x = torch.zeros(8, dtype=torch.float32, device="cuda")
    rows, cols = 64 * 1025, 1024                      # 1025 blocks x 1024 > 2^20 partial sums
    assert ((rows + 63) // 64) * cols > B.COLSUM_STATIC_MAX_FLOATS
    with pytest.raises(B.StageError) as e:
        B.dapple_colsum_static(B.DTYPE_F32, x.data_ptr(), rows, cols, cols, x.data_ptr())
    assert e.value.code == B.STAGE_E_CONFIG and "exceed" in str(e.value)
    with pytest.raises(B.StageError):
        B.dapple_colsum_static(B.DTYPE_F32, None, 64, 8, 8, x.data_ptr())
