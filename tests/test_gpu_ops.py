"""Single fused ops of the HIP library against the same contraction on the CPU in fp64."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def _rand(shape, seed, dtype):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * 0.5).to(dtype)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("n,k", [(1, 8), (5, 256), (37, 688), (1000, 1416), (4096, 4096), (130, 14336)])
def test_gemv(dtype, n, k):
    import paper_2410_12513_amd as P
    W = _rand((n, k), 1, dtype)
    x = _rand((k,), 2, torch.float32)
    y0 = _rand((n,), 3, torch.float32)
    ref = W.double() @ x.double()
    Wd, xd = W.cuda(), x.cuda()
    y = torch.empty(n, dtype=torch.float32, device="cuda")
    P.op_gemv(Wd, xd, y)
    torch.cuda.synchronize()
    scale = float((W.double().abs() @ x.double().abs()).max())
    assert float((y.cpu().double() - ref).abs().max()) <= 2e-6 * scale
    y2 = y0.cuda()
    P.op_gemv(Wd, xd, y2, accumulate=True)
    torch.cuda.synchronize()
    assert float((y2.cpu().double() - (ref + y0.double())).abs().max()) <= 2e-6 * scale + 1e-6


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("m,n,k", [(1, 1, 8), (70, 200, 136), (129, 257, 520), (300, 130, 1416), (256, 512, 1024)])
def test_gemm_nt(dtype, m, n, k):
    import paper_2410_12513_amd as P
    A = _rand((m, k), 4, dtype)
    W = _rand((n, k), 5, dtype)
    C0 = _rand((m, n), 6, torch.float32)
    ref = A.double() @ W.double().T
    Ad, Wd = A.cuda(), W.cuda()
    Cd = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    P.op_gemm_nt(Ad, Wd, Cd)
    torch.cuda.synchronize()
    scale = float((A.double().abs() @ W.double().abs().T).max())
    assert float((Cd.cpu().double() - ref).abs().max()) <= 2e-6 * scale
    C2 = C0.cuda()
    P.op_gemm_nt(Ad, Wd, C2, accumulate=True)
    torch.cuda.synchronize()
    assert float((C2.cpu().double() - (ref + C0.double())).abs().max()) <= 2e-6 * scale + 1e-6


def test_bad_arguments_are_rejected():
    import paper_2410_12513_amd as P
    W = torch.zeros((4, 12), dtype=torch.float32, device="cuda")      # k not a multiple of 8
    x = torch.zeros(12, dtype=torch.float32, device="cuda")
    y = torch.zeros(4, dtype=torch.float32, device="cuda")
    with pytest.raises(P.FirstError) as e:
        P.op_gemv(W, x, y)
    assert e.value.code == -1


@pytest.mark.parametrize("m,n,k", [(1, 1, 8), (70, 200, 136), (129, 257, 520), (300, 130, 1416)])
def test_gemm_nt_fp32_activations_split_precision(m, n, k):
    """fp32 activations against bf16 weights: the hi/lo split must recover ~16 bits of A."""
    import paper_2410_12513_amd as P
    A = _rand((m, k), 7, torch.float32)
    W = _rand((n, k), 8, torch.bfloat16)
    ref = A.double() @ W.double().T
    Cd = torch.full((m, n), float("nan"), dtype=torch.float32, device="cuda")
    P.op_gemm_nt_f32a(A.cuda(), W.cuda(), Cd)
    torch.cuda.synchronize()
    scale = float((A.double().abs() @ W.double().abs().T).max())
    err = float((Cd.cpu().double() - ref).abs().max())
    assert err <= 1.5e-5 * scale, err / scale          # a bf16-rounded A alone would give ~2e-3
