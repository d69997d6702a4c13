"""The stage's contraction kernel on its own, against fp64 matmul of the same bf16 operands."""
import numpy as np
import pytest

from tests.helpers import rel_err, to_host64

pytestmark = pytest.mark.gpu

SHAPES = [(256, 768, 256), (256, 1376, 256), (256, 256, 688), (392, 520, 328), (8, 8, 8), (1024, 2048, 512),
          (4096, 4096, 1024), (520, 4104, 264), (4096, 22016, 136),
          # tiling plans: whole rounds of 256x256 tiles + a 128x128 tail; 256x128 tiles only; an odd number of k-tiles
          (4096, 5120, 264), (2048, 4096, 200), (4096, 4096, 96)]


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_bf16_three_modes(M, N, K):
    import torch
    import paper_2410_13333_amd as mls
    g = torch.Generator(device="cpu").manual_seed(M * 7 + N * 3 + K)
    a = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    b = torch.randn(K, N, generator=g).to(torch.bfloat16).cuda()
    r = torch.randn(M, N, generator=g).to(torch.bfloat16).cuda()
    a64, b64, r64 = to_host64(a), to_host64(b), to_host64(r)
    c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    mls.gemm(0, a, b, c)
    assert rel_err(to_host64(c), a64 @ b64) < 4e-3
    mls.gemm(0, a, b, c, r)
    assert rel_err(to_host64(c), a64 @ b64 + r64) < 4e-3
    mls.gemm(1, a, b.t().contiguous(), c)
    assert rel_err(to_host64(c), a64 @ b64) < 4e-3
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    at = a.t().contiguous()
    mls.gemm(2, at, b, acc)
    mls.gemm(2, at, b, acc)
    torch.cuda.synchronize()
    assert rel_err(to_host64(acc), 0.5 + 2 * (a64 @ b64)) < 1e-5


@pytest.mark.parametrize("M,N,K", [(4096, 4096, 64), (4096, 4096, 128), (4096, 4096, 192), (4096, 4096, 320),
                                   (4000, 4104, 448), (4096, 4096, 32), (4088, 4096, 160)])
def test_bf16_16x16x32_kernel_at_awkward_depths(M, N, K):
    """At least 256 tiles of 256x256, so that the problem runs on the 16x16x32 kernel: contraction depths of one to a
    few k-tiles (prologue with nothing behind it, rings that do not come round, a k-tile count that is no multiple of
    the loop's period), ragged last tile rows, a column remainder beside it.  K % 64 != 0 exercises only the TN form
    there; the other two then run on the 32x32x16 kernels."""
    import torch
    import paper_2410_13333_amd as mls
    g = torch.Generator(device="cpu").manual_seed(M + 3 * N + 7 * K)
    a = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    b = torch.randn(K, N, generator=g).to(torch.bfloat16).cuda()
    r = torch.randn(M, N, generator=g).to(torch.bfloat16).cuda()
    ref = to_host64(a) @ to_host64(b)
    c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    mls.gemm(0, a, b, c, r)
    assert rel_err(to_host64(c), ref + to_host64(r)) < 4e-3
    mls.gemm(1, a, b.t().contiguous(), c)
    assert rel_err(to_host64(c), ref) < 4e-3
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    at = a.t().contiguous()
    mls.gemm(2, at, b, acc)
    mls.gemm(2, at, b, acc)
    torch.cuda.synchronize()
    assert rel_err(to_host64(acc), 0.5 + 2 * ref) < 1e-5


def test_fp32_three_modes():
    import torch
    import paper_2410_13333_amd as mls
    M, N, K = 136, 200, 72
    g = torch.Generator(device="cpu").manual_seed(5)
    a, b = torch.randn(M, K, generator=g).cuda(), torch.randn(K, N, generator=g).cuda()
    ref = to_host64(a) @ to_host64(b)
    c = torch.empty(M, N, device="cuda")
    mls.gemm(0, a, b, c)
    assert rel_err(to_host64(c), ref) < 1e-6
    mls.gemm(1, a, b.t().contiguous(), c)
    assert rel_err(to_host64(c), ref) < 1e-6
    acc = torch.zeros(M, N, device="cuda")
    mls.gemm(2, a.t().contiguous(), b, acc)
    assert rel_err(to_host64(acc), ref) < 1e-6


@pytest.mark.parametrize("M,N,K", [(136, 200, 72), (8, 264, 520)])
def test_bf16_register_staged_kernel_for_operands_beyond_31_bit_offsets(M, N, K):
    """An operand whose rows lie 4 MiB apart spans more than 2 GiB, which the main kernel's 31-bit buffer offsets
    cannot address: the call runs on the register-staged kernel.  All three modes, ragged tiles."""
    import torch
    import paper_2410_13333_amd as mls
    LD = 1 << 21                                    # elements between rows: (rows + 512) * LD * 2 B >= 2^31
    g = torch.Generator(device="cpu").manual_seed(M + N + K)
    big = torch.zeros(max(M, N, K), LD, dtype=torch.bfloat16, device="cuda")

    def wide(t):                                    # t's values in the first columns of the wide buffer
        v = big[:t.shape[0], :t.shape[1]]
        v.copy_(t)
        return v
    a = torch.randn(M, K, generator=g).to(torch.bfloat16).cuda()
    b = torch.randn(K, N, generator=g).to(torch.bfloat16).cuda()
    bt = b.t().contiguous()
    r = torch.randn(M, N, generator=g).to(torch.bfloat16).cuda()
    a64, b64, r64 = to_host64(a), to_host64(b), to_host64(r)
    ref = a64 @ b64
    c = torch.empty(M, N, dtype=torch.bfloat16, device="cuda")
    mls.gemm(0, wide(a), b, c, r)                   # NN, A wide
    torch.cuda.synchronize()
    assert rel_err(to_host64(c), ref + r64) <= 4e-3
    mls.gemm(1, wide(a), bt, c)                     # NT, A wide
    torch.cuda.synchronize()
    assert rel_err(to_host64(c), ref) <= 4e-3
    mls.gemm(1, a, wide(bt), c)                     # NT, B wide
    torch.cuda.synchronize()
    assert rel_err(to_host64(c), ref) <= 4e-3
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    mls.gemm(2, wide(a.t().contiguous()), b, acc)   # TN, A wide, twice: it accumulates
    mls.gemm(2, wide(a.t().contiguous()), b, acc)
    torch.cuda.synchronize()
    assert rel_err(to_host64(acc), 0.5 + 2 * ref) <= 1e-5


def test_empty_contraction():
    """K = 0 (through the C ABI directly: the operands are valid pointers to nothing): C = R for the bf16 modes,
    C unchanged for the accumulating one."""
    import ctypes as C
    import torch
    import paper_2410_13333_amd as mls
    M, N = 264, 136
    buf = torch.ones(M, 8, dtype=torch.bfloat16, device="cuda")
    r = torch.randn(M, N, device="cuda").to(torch.bfloat16)
    c = torch.full((M, N), 7.0, dtype=torch.bfloat16, device="cuda")
    acc = torch.full((M, N), 0.5, dtype=torch.float32, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda t: C.c_void_p(t.data_ptr())
    L = mls.lib()
    assert L.mls_gemm(mls.MLS_BF16, 0, p(buf), 8, p(buf), N, p(c), N, p(r), M, N, 0, st) == 0
    torch.cuda.synchronize()
    assert torch.equal(c, r)
    assert L.mls_gemm(mls.MLS_BF16, 1, p(buf), 8, p(buf), 8, p(c), N, None, M, N, 0, st) == 0
    assert L.mls_gemm(mls.MLS_BF16, 2, p(buf), M, p(buf), N, p(acc), N, None, M, N, 0, st) == 0
    torch.cuda.synchronize()
    assert float(c.float().abs().max()) == 0.0 and float((acc - 0.5).abs().max()) == 0.0
