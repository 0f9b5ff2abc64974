"""GPU parity of the product with a symmetric operand given by one stored triangle
(gemm_epilogue_bf16_fused with a_structure = sym_lower / sym_upper) against its CPU oracle
(oracle/gemm_symm_oracle.c) on the same seeded inputs, element by element, through the C-ABI.

The unread triangle of A is filled with NaN on the device: a single element of it reaching a
product would show.  Shapes with N <= 32, M >= 512 take the kernel that fetches every stored element
once; the rest take the guarded kernel with mirrored indices."""
import numpy as np
import pytest

from paper_2604_01489_amd import binding, inputs as gen

from gpu_util import CANARY, compare, to_device, torch_device

pytestmark = pytest.mark.gpu

NAN_BITS = np.uint16(0x7FC0)


def run_symm_case(oracle, M, N, *, uplo="lower", batch=1, transB=False, alpha=0.5, with_bias=True, with_row_scale=False,
                  residual=None, beta=0.75, act="none", clamp=None, out="f32", pad=(0, 0, 0), seed=0, workspace=False,
                  misalign=0, scale=None):
    """``pad`` = extra elements on (lda, ldb, ldc); ``workspace``: pass a caller's workspace of the size the
    library asks for.  Returns (got, configuration name)."""
    import torch
    lda = M + pad[0]
    rowsB, colsB = (N, M) if transB else (M, N)
    ldb, ldc = colsB + pad[1], N + pad[2]
    scale = M ** -0.5 if scale is None else scale
    A = gen.to_bf16_bits(gen.normal(seed, gen.STREAM_A, batch * M * M, scale).reshape(batch, M, M))
    B = gen.to_bf16_bits(gen.normal(seed, gen.STREAM_B, batch * M * N, 1.0).reshape(batch, M, N))
    bias = gen.uniform(seed, gen.STREAM_BIAS, N, -1.0, 1.0) if with_bias else None
    rs = gen.uniform(seed, 7, M, 0.25, 2.0) if with_row_scale else None
    # the array as the caller holds it: the stored triangle, NaN everywhere else (other triangle and padding)
    As = np.full((batch, M, lda), NAN_BITS, dtype=np.uint16)
    keep = np.tri(M, dtype=bool) if uplo == "lower" else np.tri(M, dtype=bool).T
    As[:, :, :M] = np.where(keep[None], A, NAN_BITS)
    Bs = np.full((batch, rowsB, ldb), np.uint16(0x7F00), dtype=np.uint16)
    Bs[:, :, :colsB] = B.transpose(0, 2, 1) if transB else B
    Rs = None
    if residual is not None:
        R32 = gen.uniform(seed, 8, batch * M * N, -1.0, 1.0).reshape(batch, M, N)
        Rs = gen.to_bf16_bits(R32) if residual == "bf16" else R32

    def shifted(flat):
        buf = np.full(flat.size + misalign, np.uint16(0x7F00), dtype=np.uint16)
        buf[misalign:] = flat
        t = to_device(buf)
        return t, t[misalign:]

    keepA, dA = shifted(As.ravel())
    keepB, dB = shifted(Bs.ravel())
    dbias, drs, dR = to_device(bias), to_device(rs), to_device(None if Rs is None else Rs.ravel())
    if dR is not None and residual == "bf16":
        dR = dR.view(torch.bfloat16)
    cdtype = torch.float32 if out == "f32" else torch.bfloat16
    canary = CANARY if out == "f32" else -7.0e30
    dC = torch.full((batch * M * ldc,), canary, dtype=cdtype, device=torch_device())
    structure = "sym_" + uplo
    ws = None
    if workspace:
        args = binding.fused_args(M, N, M, dA.data_ptr(), lda, dB.data_ptr(), ldb, dC.data_ptr(), ldc, batch=batch, transB=transB,
                                  c_type="f32" if out == "f32" else "bf16", a_structure=structure)
        need = binding.fused_workspace_bytes(args)
        assert need > 0
        ws = torch.empty(need // 4, dtype=torch.float32, device=torch_device())
    print(f"symm case M={M} N={N} uplo={uplo} batch={batch} tB={transB} pad={pad} act={act} out={out} res={residual} "
          f"rs={with_row_scale} clamp={clamp} workspace={workspace} misalign={misalign}", flush=True)
    binding.gemm_epilogue_bf16_fused(M, N, M, dA, lda, dB, ldb, dC, ldc, batch=batch, transB=transB, alpha=alpha,
                                     row_scale=drs, bias=dbias, residual=dR, ldr=N, beta=beta, act=act, clamp=clamp,
                                     a_structure=structure, workspace=ws)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    outv = dC.to(torch.float32).cpu().numpy().reshape(batch, M, ldc)
    canary32 = np.float32(torch.tensor(canary, dtype=cdtype).to(torch.float32).item())
    assert np.all(outv[:, :, N:] == canary32), f"{cfg}: wrote into the padding of C"
    got = outv[:, :, :N]
    assert np.all(np.isfinite(got)), f"{cfg}: an element of the unread triangle reached the result"
    ref = oracle.gemm_symm(M, N, As, Bs, uplo=uplo, batch=batch, transB=transB, lda=lda, ldb=ldb, alpha=alpha,
                           row_scale=rs, bias=bias, residual=Rs, ldr=N, beta=beta, act=act, clamp=clamp, out=out)
    compare(got, ref, f"{cfg} symm {M}x{N}x{batch}", bf16_out=(out == "bf16"))
    del keepA, keepB
    return got, cfg


@pytest.mark.parametrize("uplo", ["lower", "upper"])
def test_symm_few_columns_every_element_once(oracle, uplo):
    """The kernel for few output columns: one super-tile and several, 256 and 512 wide, ragged last
    super-tile, N of one column to 32, both column widths of the small operand's image."""
    for M, N, kw in [(512, 16, {}), (1024, 8, dict(pad=(8, 0, 3))), (1288, 32, dict(act="gelu_tanh")),
                     (2048, 1, dict(with_bias=False)), (1536, 24, dict(act="relu", clamp=(0.0, 0.4)))]:
        _, cfg = run_symm_case(oracle, M, N, uplo=uplo, seed=M + N, **kw)
        assert cfg.startswith(f"bf16_symm_{uplo}_"), cfg


@pytest.mark.parametrize("uplo", ["lower", "upper"])
def test_symm_chain_batches_and_storage_of_b(oracle, uplo):
    """The whole consumer chain behind the symmetric product, bf16 and fp32 output, B stored either way round
    (16-byte pieces of B where it allows them, single elements otherwise), batches, a caller's workspace."""
    run_symm_case(oracle, 640, 16, uplo=uplo, batch=3, with_row_scale=True, residual="bf16", act="relu", clamp=(0.0, 6.0),
                  out="bf16", seed=5)
    run_symm_case(oracle, 768, 12, uplo=uplo, transB=True, residual="f32", act="gelu_tanh", pad=(16, 5, 1), seed=6)
    run_symm_case(oracle, 1024, 32, uplo=uplo, batch=2, transB=True, pad=(0, 8, 0), workspace=True, seed=7)
    run_symm_case(oracle, 520, 8, uplo=uplo, pad=(0, 3, 0), workspace=True, seed=8)          # B rows not in 16-byte pieces


def test_symm_wide_super_tiles(oracle):
    """Large matrices: the width of the super-tiles follows the number of rounds their workgroups take on
    the CUs and the bytes of partial results (the library's own choice is asserted): 768 at 16384 with 16
    columns (253 workgroups, one round), 512 with 32 columns there, 256 at 12288; ragged at 12296."""
    _, cfg = run_symm_case(oracle, 16384, 16, act="relu", seed=20)
    assert cfg == "bf16_symm_lower_768x768_n16", cfg
    _, cfg = run_symm_case(oracle, 16384, 32, uplo="upper", seed=23)
    assert cfg == "bf16_symm_upper_512x512_n32", cfg
    _, cfg = run_symm_case(oracle, 12288, 4, seed=21)
    assert cfg == "bf16_symm_lower_256x256_n16", cfg
    _, cfg = run_symm_case(oracle, 12296, 16, uplo="upper", act="relu", seed=22)
    assert cfg.startswith("bf16_symm_upper_"), cfg


@pytest.mark.parametrize("uplo", ["lower", "upper"])
def test_symm_guarded_kernel(oracle, uplo):
    """Argument lists the kernel for few columns does not take: many columns, small or odd M, unaligned
    pointers; with and without K slices."""
    for M, N, kw in [(100, 40, {}), (300, 64, dict(act="gelu_tanh", batch=2)), (515, 16, dict(pad=(1, 0, 0))),
                     (1024, 16, dict(misalign=1)), (256, 8, dict(out="bf16", residual="f32"))]:
        _, cfg = run_symm_case(oracle, M, N, uplo=uplo, seed=3 * M + N, **kw)
        assert cfg.startswith("bf16_fused_generic"), cfg


def test_symm_is_repeatable_and_agrees_with_the_dense_call(oracle):
    """Bit for bit the same on a second call; and within rounding of the general call on the explicitly
    mirrored matrix (another order of additions)."""
    import torch
    a, cfg = run_symm_case(oracle, 1024, 16, seed=31)
    b, _ = run_symm_case(oracle, 1024, 16, seed=31)
    assert np.array_equal(a, b)
    M, N = 1024, 16
    A = gen.to_bf16_bits(gen.normal(31, gen.STREAM_A, M * M, M ** -0.5).reshape(M, M))
    S = np.where(np.tri(M, dtype=bool), A, A.T)
    B = gen.to_bf16_bits(gen.normal(31, gen.STREAM_B, M * N, 1.0).reshape(M, N))
    bias = gen.uniform(31, gen.STREAM_BIAS, N, -1.0, 1.0)
    C = torch.empty(M, N, dtype=torch.float32, device=torch_device())
    binding.gemm_epilogue_bf16_fused(M, N, M, to_device(S), M, to_device(B), N, C, N, alpha=0.5, bias=to_device(bias))
    torch.cuda.synchronize()
    dense = C.cpu().numpy().astype(np.float64)
    assert np.linalg.norm(dense - a[0]) <= 1e-5 * np.linalg.norm(dense)


def test_symm_argument_errors():
    P = 0x10000
    ok = dict(M=64, N=8, K=64, A_ptr=P, lda=64, B_ptr=P, ldb=8, C_ptr=P, ldc=8, a_structure="sym_lower")

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        pos = [a.pop(k) for k in ("M", "N", "K", "A_ptr", "lda", "B_ptr", "ldb", "C_ptr", "ldc")]
        return binding.raw_fused(binding.fused_args(*pos, **a))

    assert call(K=32, lda=64) == 2          # a symmetric operand is square
    assert call(transA=True) == 8           # its transposed storage is the other triangle: say that instead
    assert call(a_structure=5) == 8
