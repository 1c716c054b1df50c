"""The allocation-free product entry point against the allocating one it is a variant of.

eesd_op_gemm_noalloc stages the bf16 activation rows in a fixed device array of the library; its kernels
are the ones eesd_op_gemm launches, so the two results must be bit-identical - on a first call and on a
second, smaller one that finds the array full of the first call's rows.  (Collected last: see the file name.)
"""
import numpy as np
import pytest
import torch

from gpu_common import require_gpu

pytestmark = pytest.mark.gpu


def _pair(out, inn, M, seed, layout):
    import paper_2406_03853_amd as pk
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    W = (torch.randn(out, inn, device="cuda", generator=g) * 0.02).to(torch.bfloat16)
    X = torch.randn(M, inn, device="cuda", generator=g)
    Wd = pk.pack_weight(W) if layout == pk.WEIGHTS_TILED else W
    Y0 = torch.full((M, out), float("nan"), device="cuda")
    Y1 = torch.full((M, out), float("nan"), device="cuda")
    pk.op_gemm(Wd, X, Y0, pk.GEMM_MFMA, weight_layout=layout)
    pk.op_gemm_noalloc(Wd, X, Y1, weight_layout=layout)
    torch.cuda.synchronize()
    ref = X.to(torch.bfloat16).double() @ W.double().t()
    return Y0.cpu().numpy(), Y1.cpu().numpy(), ref.cpu().numpy()


@pytest.mark.parametrize("layout", [0, 1])
def test_noalloc_product_equals_the_allocating_one_on_two_calls_in_a_row(layout):
    require_gpu()
    # first call: 16 rows x 13824 columns fill the staging array; second: fewer rows, fewer columns, another matrix shape
    # (5120 x 13824 is dealt to one row group per CU in the tile-major layout, 2048 x 1024 keeps one tile per group)
    for out, inn, M, seed in ((5120, 13824, 16, 1), (2048, 1024, 3, 2)):
        y0, y1, ref = _pair(out, inn, M, seed, layout)
        assert np.isfinite(y1).all()
        assert np.array_equal(y0, y1), (out, inn, M)
        assert np.max(np.abs(y1 - ref)) <= 1e-3 * np.max(np.abs(ref))     # and both are the product itself (fp32 accumulation of bf16 operands)


def test_noalloc_rejects_sizes_beyond_the_fixed_array():
    require_gpu()
    import paper_2406_03853_amd as pk
    W = torch.zeros(64, 128, device="cuda", dtype=torch.bfloat16)
    Y = torch.zeros(17, 64, device="cuda")
    with pytest.raises(pk.EesdError) as e:
        pk.op_gemm_noalloc(W, torch.zeros(17, 128, device="cuda"), Y)          # 17 rows
    assert e.value.code == -4
    Wbig = torch.zeros(16, 32768 + 128, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(pk.EesdError) as e:
        pk.op_gemm_noalloc(Wbig, torch.zeros(1, 32768 + 128, device="cuda"), torch.zeros(1, 16, device="cuda"))   # too many columns
    assert e.value.code == -4
