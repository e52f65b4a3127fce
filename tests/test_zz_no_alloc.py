"""The GEMM entry point that allocates nothing (sjd_op_gemm_static: temporaries in a workspace that is part of the
library image) against the allocating one (sjd_op_gemm), through the C ABI: same kernels and plan, so the results
must be identical bit for bit; and against double-precision numpy on the rounded operands.  Two calls in a row, the
second smaller, so that what the first left in the shared workspace would show."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _operands(M, N, K, dtype, seed):
    import torch
    rng = np.random.default_rng(seed)
    td = torch.float32 if dtype == "f32" else torch.bfloat16
    A = torch.from_numpy(rng.standard_normal((M, K)).astype(np.float32)).cuda().to(td)
    W = torch.from_numpy((rng.standard_normal((N, K)) * 0.05).astype(np.float32)).cuda().to(td)
    return A, W


@pytest.mark.parametrize("dtype,first,second", [("bf16", (96, 2080, 512, 0), (33, 130, 256, 3)),
                                                 ("bf16", (512, 1024, 1024, 0), (7, 100, 64, 0)),
                                                 ("f32", (33, 130, 1024, 0), (7, 100, 64, 0))])
def test_static_gemm_equals_the_allocating_one_twice_in_a_row(dtype, first, second):
    import paper_2512_07503_amd as sjd
    for i, (M, N, K, splits) in enumerate((first, second)):
        A, W = _operands(M, N, K, dtype, 17 * M + N + i)
        want, _ = sjd.op_gemm(A, W, splits=splits)
        rc, got = sjd.op_gemm_static(A, W, splits=splits)
        assert rc == sjd.OK, (rc, sjd.lib().sjd_last_error(None))
        assert np.array_equal(got.cpu().numpy().view(np.uint32), want.cpu().numpy().view(np.uint32)), (dtype, M, N, K)
        exact = A.double().cpu().numpy() @ W.double().cpu().numpy().T
        assert np.abs(got.cpu().numpy() - exact).max() < 2e-5 * np.abs(exact).max() * max(1.0, np.sqrt(K / 256))


def test_static_gemm_refuses_sizes_beyond_its_workspace():
    import paper_2512_07503_amd as sjd
    A, W = _operands(64, 8192, 4096, "bf16", 3)      # 64 MiB of weights alone
    rc, _ = sjd.op_gemm_static(A, W)
    assert rc == sjd.ECAPACITY
    assert b"static workspace" in sjd.lib().sjd_last_error(None)
    A, W = _operands(32, 256, 128, "bf16", 4)        # ... and the library still works afterwards
    want, _ = sjd.op_gemm(A, W)
    rc, got = sjd.op_gemm_static(A, W)
    assert rc == sjd.OK and np.array_equal(got.cpu().numpy(), want.cpu().numpy())
