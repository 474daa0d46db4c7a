"""GPU test of the entry point that allocates nothing (nvfp4_gemm_nt_static): same bytes as nvfp4_gemm_nt.

The static entry point runs the same kernels with the library's static device array in place of the caller's
workspace, so its output must equal nvfp4_gemm_nt's bit for bit.  Two calls in a row share the array, the second
on a smaller product (the array then still holds the first call's partial sums); a product that needs no scratch
and one that needs more than the array holds are covered too.
"""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


def _operand(tj, rows, K, seed):
    bits = wl.normal_bf16((rows, K), 1.0, seed, 1e-3, 50.0)
    x = torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)
    return tj.quantize(x, 0, tj.binding.ROUND_RTN)


@pytest.mark.parametrize("out_dtype", [0, 1])
def test_static_scratch_product_equals_workspace_product(out_dtype):
    import paper_2510_27527_amd as tj
    B = tj.binding
    B.lib()
    # (M, N, K): a split reduction, then a smaller split reduction, then a product without scratch
    shapes = [(768, 768, 8192), (256, 512, 4096), (512, 384, 512)]
    assert B.workspace_bytes(B.OP_GEMM, 768, 8192, 768) > B.workspace_bytes(B.OP_GEMM, 256, 4096, 512) > 0
    assert B.workspace_bytes(B.OP_GEMM, 512, 512, 384) == 0
    jobs = []
    for i, (M, N, K) in enumerate(shapes):
        A, Bt = _operand(tj, M, K, 900 + 2 * i), _operand(tj, N, K, 901 + 2 * i)
        ref = tj.gemm_nt(A, Bt, out_dtype)
        out = torch.full((M, N), float("nan"), dtype=ref.dtype, device="cuda")
        jobs.append((A, Bt, ref, out))
    torch.cuda.synchronize()
    for A, Bt, ref, out in jobs:                     # back to back on one stream, no synchronisation in between
        print("static product %d x %d x %d" % (A.rows, Bt.rows, A.K), flush=True)
        tj.gemm_nt_static(A, Bt, out, out_dtype)
    torch.cuda.synchronize()
    for A, Bt, ref, out in jobs:
        assert torch.equal(out, ref), (A.rows, Bt.rows, A.K)
    # once more in the other order: the small product first, the large one over its leftovers
    for A, Bt, ref, out in reversed(jobs):
        out.fill_(float("nan"))
        tj.gemm_nt_static(A, Bt, out, out_dtype)
    torch.cuda.synchronize()
    for A, Bt, ref, out in jobs:
        assert torch.equal(out, ref), (A.rows, Bt.rows, A.K)


def test_static_scratch_rejects_what_does_not_fit():
    import paper_2510_27527_amd as tj
    B = tj.binding
    M, N, K = 3072, 3072, 65536
    assert B.workspace_bytes(B.OP_GEMM, M, K, N) > B.STATIC_SCRATCH_BYTES
    A, Bt = tj.alloc_nvfp4(M, K), tj.alloc_nvfp4(N, K)
    out = torch.zeros((M, N), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.NVFP4Error) as e:
        tj.gemm_nt_static(A, Bt, out)
    assert e.value.code == B.ERR_SCRATCH
    torch.cuda.synchronize()
    assert not out.any()                             # nothing was enqueued
