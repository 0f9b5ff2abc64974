"""Operands beyond 4 GiB: byte offsets past 2^32 and element offsets past 2^31 (row offsets, batch strides).
The large operand is drawn on the device by torch's seeded generator (it is an input, not a result of the
library), the oracle gets the sampled rows copied back, and every sampled output row is compared."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

REL_FRO_TOL, ELEM_TOL = 1e-3, 1e-2


def _big_bf16(rows, cols, seed, scale):
    import torch
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    out = torch.empty(rows, cols, dtype=torch.bfloat16, device="cuda:0")
    step = max(1, (1 << 28) // cols)                       # rows per chunk: 2^28 fp32 temporaries at most
    for r0 in range(0, rows, step):
        r1 = min(rows, r0 + step)
        out[r0:r1] = (torch.randn(r1 - r0, cols, generator=g, device="cuda:0") * scale).to(torch.bfloat16)
    return out


def _bits(t):
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def _rows(M):
    return np.unique(np.concatenate([np.arange(32), M // 2 + np.arange(-16, 16), (1 << 20) + np.arange(8) if M > (1 << 20) + 8
                                     else np.arange(0), M - 32 + np.arange(32)]))


def _check(got, ref, what):
    err = np.abs(got - ref)
    assert np.all(np.isfinite(got)), what
    assert np.all(err <= ELEM_TOL * np.maximum(1.0, np.abs(ref))), f"{what}: element {np.unravel_index(int(np.argmax(err)), err.shape)}"
    rel = float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300))
    assert rel <= REL_FRO_TOL, f"{what}: relative Frobenius error {rel:.3e}"
    return rel


def test_plain_a_of_five_gigabytes(oracle):
    """A is 1.2 M x 2048 bf16 (4.9 GB): the last tile rows start 4.9e9 bytes into it."""
    import torch
    from paper_2604_01489_amd import binding
    M, N, K = 1_200_000, 64, 2048
    A = _big_bf16(M, K, 101, K ** -0.5)
    B = _big_bf16(K, N, 102, 1.0)
    bias = torch.linspace(-0.5, 0.5, N, device="cuda:0")
    C = torch.empty(M, N, dtype=torch.float32, device="cuda:0")
    print(f"large plain case M={M} N={N} K={K}", flush=True)
    binding.gemm_epilogue_bf16(M, N, K, A, K, B, N, bias, 0.5, "relu", C, N, 1)
    torch.cuda.synchronize()
    rows = _rows(M)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.gemm_epilogue(_bits(A[idx]), _bits(B), bias.cpu().numpy(), 0.5, "relu")
    _check(C[idx].cpu().numpy().astype(np.float64), ref, f"plain {M}x{N}x{K} [{binding.last_config()}]")


def test_four_wave_kernel_a_of_five_gigabytes(oracle):
    """The same A against 256 columns, both storages of B: 4688 tile rows of the four-wave kernel (the last one
    ragged), tile bases up to 4.9e9 bytes into A, fp32 and bf16 output."""
    import torch
    from paper_2604_01489_amd import binding
    M, N, K = 1_200_000, 256, 2048
    A = _big_bf16(M, K, 111, K ** -0.5)
    B = _big_bf16(K, N, 112, 1.0)
    bias = torch.linspace(-0.5, 0.5, N, device="cuda:0")
    C = torch.empty(M, N, dtype=torch.float32, device="cuda:0")
    print(f"large four-wave case M={M} N={N} K={K}", flush=True)
    binding.gemm_epilogue_bf16(M, N, K, A, K, B, N, bias, 0.5, "relu", C, N, 1)
    torch.cuda.synchronize()
    assert binding.last_config() == "bf16_256x256x64_w4"
    rows = _rows(M)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.gemm_epilogue(_bits(A[idx]), _bits(B), bias.cpu().numpy(), 0.5, "relu")
    _check(C[idx].cpu().numpy().astype(np.float64), ref, f"plain {M}x{N}x{K} [{binding.last_config()}]")
    del C
    Bt = B.t().contiguous()
    C16 = torch.empty(M, N, dtype=torch.bfloat16, device="cuda:0")
    binding.gemm_epilogue_bf16_fused(M, N, K, A, K, Bt, K, C16, N, transB=True, alpha=0.5, bias=bias, act="relu")
    torch.cuda.synchronize()
    assert binding.last_config() == "bf16_fused_256x256x64_w4_nt"
    got = C16[idx].to(torch.float32).cpu().numpy().astype(np.float64)
    # the oracle's fp32-output result rounded as the kernel rounds: compare within the bar plus half a bf16 step
    err = np.abs(got - ref)
    assert np.all(err <= ELEM_TOL * np.maximum(1.0, np.abs(ref)) + np.abs(ref) * 2.0 ** -8), "bf16 output"
    assert float(np.linalg.norm(got - ref) / np.linalg.norm(ref)) <= 4e-3


@pytest.mark.parametrize("transA", [False, True])
def test_fused_batch_stride_past_two_to_the_31(oracle, transA):
    """Two batches of a 70000 x 32768 A (2.29e9 elements each, 9.2 GB together), stored either way round,
    weights N x K, bf16 out: the second batch starts past 2^31 elements."""
    import torch
    from paper_2604_01489_amd import binding
    batch, M, N, K = 2, 70000, 64, 32768
    rowsA, colsA = (K, M) if transA else (M, K)
    A = _big_bf16(batch * rowsA, colsA, 201 + transA, K ** -0.5).view(batch, rowsA, colsA)
    W = _big_bf16(batch * N, K, 203, 1.0).view(batch, N, K)
    bias = torch.linspace(-0.5, 0.5, N, device="cuda:0")
    C = torch.empty(batch, M, N, dtype=torch.bfloat16, device="cuda:0")
    print(f"large fused case batch={batch} M={M} N={N} K={K} transA={transA}", flush=True)
    binding.gemm_epilogue_bf16_fused(M, N, K, A, colsA, W, K, C, N, batch=batch, transA=transA, transB=True, alpha=0.5,
                                     bias=bias, act="relu")
    torch.cuda.synchronize()
    cfg = binding.last_config()
    rows = _rows(M)
    idx = torch.from_numpy(rows).cuda()
    A_s = A[:, :, idx] if transA else A[:, idx]
    ref = oracle.gemm_fused(len(rows), N, K, _bits(A_s), _bits(W), batch=batch, transA=transA, transB=True, alpha=0.5,
                            bias=bias.cpu().numpy(), act="relu", out="bf16")
    _check(C[:, idx].to(torch.float32).cpu().numpy().astype(np.float64), ref, f"fused batch stride [{cfg}]")


def test_rowsum_input_of_five_gigabytes(oracle):
    import torch
    from paper_2604_01489_amd import binding
    M, N, K = 1_200_000, 512, 2048
    A = _big_bf16(M, K, 301, K ** -0.5)
    W = _big_bf16(N, K, 302, 1.0)
    bias = torch.linspace(-0.5, 0.5, N, device="cuda:0")
    params = torch.empty(K + 1, dtype=torch.float32, device="cuda:0")
    y = torch.empty(M, dtype=torch.float32, device="cuda:0")
    print(f"large rowsum case M={M} N={N} K={K}", flush=True)
    binding.gemm_rowsum_params_bf16(N, K, W, K, True, bias, params)
    binding.gemm_rowsum_bf16(M, K, A, K, params, 0.5, y)
    torch.cuda.synchronize()
    rows = _rows(M)
    idx = torch.from_numpy(rows).cuda()
    ref = oracle.gemm_rowsum(_bits(A[idx]), np.ascontiguousarray(_bits(W).T), bias.cpu().numpy(), 0.5)
    _check(y[idx].cpu().numpy().astype(np.float64), ref, "rowsum 1.2M rows")


@pytest.mark.parametrize("images,expect", [(15, "conv_bf16_128x128x32_w4"), (17, "conv_bf16_generic_64x64x32")])
def test_conv_input_around_two_gigabytes(oracle, images,expect):
    """The gathering kernel addresses the input with 31-bit byte offsets: an input just under 2 GiB takes it
    (3x3 taps reach the last bytes), one just over takes the guarded kernel.  First and last image compared."""
    import torch
    from paper_2604_01489_amd import binding
    H = W = 512
    Cin, Cout, KH = 256, 32, 3 if images == 15 else 1
    X = _big_bf16(images * H * W, Cin, 400 + images, 1.0).view(images, H, W, Cin)
    Wt = _big_bf16(Cout * KH * KH, Cin, 401, (KH * KH * Cin) ** -0.5).view(Cout, KH, KH, Cin)
    bias = torch.linspace(-0.5, 0.5, Cout, device="cuda:0")
    Y = torch.empty(images, H, W, Cout, dtype=torch.bfloat16, device="cuda:0")
    print(f"large conv case images={images} {H}x{W}x{Cin} -> {Cout}, {KH}x{KH}", flush=True)
    binding.conv2d_epilogue_bf16(X, Wt, Y, pad=(KH // 2, KH // 2), bias=bias, act="relu")
    torch.cuda.synchronize()
    assert binding.last_config() == expect
    for img in (0, images - 1):
        ref = oracle.conv2d_nhwc(_bits(X[img:img + 1]), _bits(Wt), pad=(KH // 2, KH // 2), bias=bias.cpu().numpy(),
                                 act="relu", out="bf16")
        _check(Y[img:img + 1].to(torch.float32).cpu().numpy().astype(np.float64), ref, f"conv image {img} of {images}")
