"""The matrix-product kernels alone, through the C ABI (mslt_debug_gemm), against the plain
definition C = A B^T evaluated in float64 on the same bf16-rounded operands: every operand
layout (forward, data-gradient, weight-gradient form), every tile shape, split-k, sizes that span
several tiles with odd numbers of k tiles."""
import numpy as np
import pytest

from paper_2011_13635_amd import binding, synth

pytestmark = pytest.mark.gpu


def _operands(torch, M, N, K, akc, bkc, seed):
    # values of a few bf16 digits: their products and partial sums stay exact in fp32 for a long time
    a = ((synth.rand_u64(seed, 11, np.arange(M * K)) % 33).astype(np.float64) - 16.0) / 16.0
    b = ((synth.rand_u64(seed, 12, np.arange(N * K)) % 33).astype(np.float64) - 16.0) / 16.0
    A = a.reshape(M, K)
    B = b.reshape(N, K)
    ref = A @ B.T
    dev = "cuda:0"
    ta = torch.tensor(A if akc else A.T.copy(), dtype=torch.float32).to(torch.bfloat16).contiguous().to(dev)
    tb = torch.tensor(B if bkc else B.T.copy(), dtype=torch.float32).to(torch.bfloat16).contiguous().to(dev)
    return ta, tb, ref


CASES = []
for akc, bkc in ((1, 1), (1, 0), (0, 0), (0, 1)):
    CASES.append((1, 0, 0, 64, akc, bkc, 1))        # 128-wide kernel, tile height chosen by shape
    CASES.append((1, 256, 0, 64, akc, bkc, 2))
    for tm, tn in ((256, 256), (256, 128), (128, 256), (128, 128)):
        CASES.append((2, tm, tn, 64, akc, bkc, 1))
        CASES.append((2, tm, tn, 64, akc, bkc, 3))
    CASES.append((2, 256, 256, 32, akc, bkc, 1))
    CASES.append((2, 256, 128, 32, akc, bkc, 2))


@pytest.mark.parametrize("kernel,tm,tn,tk,akc,bkc,splitk", CASES)
def test_product_equals_plain_definition(kernel, tm, tn, tk, akc, bkc, splitk):
    import torch
    M, N, K = 512, 768, 704          # 2 x 3 tiles of 256, 11 k tiles of 64
    ta, tb, ref = _operands(torch, M, N, K, akc, bkc, seed=5 + 2 * akc + bkc)
    partials = torch.zeros(splitk * M * N, dtype=torch.float32, device="cuda:0") if splitk > 1 else None
    for out_dtype, tol in ((torch.float32, 1e-6), (torch.bfloat16, 2.0 ** -8)):
        c = torch.full((M, N), float("nan"), dtype=out_dtype, device="cuda:0")
        binding.mslt_debug_gemm(ta, tb, c, M, N, K, akc, bkc, kernel, tm, tn, tk, splitk, partials)
        torch.cuda.synchronize()
        got = c.to(torch.float64).cpu().numpy()
        scale = np.abs(ref).max()
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= tol * scale, (np.abs(got - ref).max(), scale)


def test_guarded_kernel_takes_ragged_shapes_and_agrees():
    import torch
    M, N, K = 130, 70, 45
    for akc, bkc in ((1, 1), (1, 0), (0, 0)):
        ta, tb, ref = _operands(torch, M, N, K, akc, bkc, seed=9)
        c = torch.zeros((M, N), dtype=torch.float32, device="cuda:0")
        binding.mslt_debug_gemm(ta, tb, c, M, N, K, akc, bkc, 0)
        torch.cuda.synchronize()
        assert np.abs(c.cpu().numpy() - ref).max() <= 1e-6 * np.abs(ref).max()


def test_unsupported_choices_are_refused_without_work():
    import torch
    ta, tb, _ = _operands(torch, 256, 256, 128, 1, 1, seed=3)
    c = torch.zeros((256, 256), dtype=torch.float32, device="cuda:0")
    for args in ((2, 256, 192, 64, 1), (2, 128, 128, 32, 1), (1, 64, 0, 64, 1), (2, 256, 256, 64, 4), (3, 0, 0, 64, 1)):
        with pytest.raises(binding.MsltError) as ei:
            binding.mslt_debug_gemm(ta, tb, c, 256, 256, 128, 1, 1, args[0], args[1], args[2], args[3], args[4])
        assert ei.value.code == binding.MSLT_ERR_ARG
    torch.cuda.synchronize()
    assert float(c.abs().max()) == 0.0
