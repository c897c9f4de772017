"""Population-batched bf16 MFMA GEMM against the plain definition (numpy float64 matmul of the
same bf16-rounded operands), all four operand layouts, several tiles and ragged tails."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _bf16_round(x):
    import torch
    return torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16)


@pytest.mark.parametrize("M,N,K,batch", [(128, 128, 64, 2), (200, 136, 72, 3), (40, 264, 1024, 2), (1, 8, 8, 1),
                                         (300, 130, 100, 2), (300, 130, 128, 2), (672, 264, 512, 3), (512, 512, 1056, 64),
                                         (256, 768, 1024, 86), (512, 512, 600, 48)])
@pytest.mark.parametrize("a_m_contig", [0, 1])
@pytest.mark.parametrize("b_k_contig", [0, 1])
@pytest.mark.parametrize("out_bf16", [False, True])
def test_batched_gemm(M, N, K, batch, a_m_contig, b_k_contig, out_bf16):
    import torch
    from paper_1711_09846_amd import binding
    rng = np.random.default_rng(M * 7 + N * 3 + K + batch)
    pad = lambda v: (v + 7) // 8 * 8
    A = _bf16_round(rng.standard_normal((batch, M, K)))
    B = _bf16_round(rng.standard_normal((batch, K, N)))
    ref = np.matmul(A.to(torch.float64).numpy(), B.to(torch.float64).numpy())
    if a_m_contig:
        lda = pad(M) + 8
        a_mem = torch.zeros(batch, K, lda, dtype=torch.bfloat16)
        a_mem[:, :, :M] = A.transpose(1, 2)
        sa = K * lda
    else:
        lda = pad(K) + 8
        a_mem = torch.zeros(batch, M, lda, dtype=torch.bfloat16)
        a_mem[:, :, :K] = A
        sa = M * lda
    if b_k_contig:
        ldb = pad(K)
        b_mem = torch.zeros(batch, N, ldb, dtype=torch.bfloat16)
        b_mem[:, :, :K] = B.transpose(1, 2)
        sb = N * ldb
    else:
        ldb = pad(N)
        b_mem = torch.zeros(batch, K, ldb, dtype=torch.bfloat16)
        b_mem[:, :, :N] = B
        sb = K * ldb
    ldc = N + 3
    c = torch.full((batch, M, ldc), 7.0, dtype=torch.bfloat16 if out_bf16 else torch.float32, device="cuda")
    a_d, b_d = a_mem.cuda(), b_mem.cuda()
    binding.batched_gemm_bf16(a_d, b_d, c, M, N, K, batch, lda, sa, a_m_contig, ldb, sb, b_k_contig, ldc, M * ldc)
    torch.cuda.synchronize()
    got = c.cpu().to(torch.float64).numpy()
    assert np.all(got[:, :, N:] == 7.0)                       # nothing written past the row
    scale = np.matmul(np.abs(A.to(torch.float64).numpy()), np.abs(B.to(torch.float64).numpy()))
    tol = 2 ** -8 if out_bf16 else 1e-5
    assert np.max(np.abs(got[:, :, :N] - ref) / (scale + 1e-30)) <= tol


def test_shared_operand_stride_zero():
    import torch
    from paper_1711_09846_amd import binding
    rng = np.random.default_rng(1)
    A = _bf16_round(rng.standard_normal((256, 64)))
    B = _bf16_round(rng.standard_normal((3, 64, 128)))
    c = torch.zeros(3, 256, 128, dtype=torch.float32, device="cuda")
    binding.batched_gemm_bf16(A.cuda(), B.cuda(), c, 256, 128, 64, 3, 64, 0, 0, 128, 64 * 128, 0, 128, 256 * 128)
    ref = np.matmul(A.to(torch.float64).numpy()[None], B.to(torch.float64).numpy())
    assert np.max(np.abs(c.cpu().numpy() - ref)) < 1e-4


def test_gemm_rejects_bad_arguments():
    import torch
    from paper_1711_09846_amd import binding
    a = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(64, 64, dtype=torch.float32, device="cuda")
    with pytest.raises(binding.PbtError):
        binding.batched_gemm_bf16(a, a, c, 64, 64, 64, 1, 60, 0, 0, 64, 0, 0, 64, 0)     # pitch not multiple of 8
    with pytest.raises(binding.PbtError):
        binding.batched_gemm_bf16(a, a, c, 0, 64, 64, 1, 64, 0, 0, 64, 0, 0, 64, 0)      # empty M
