"""Helpers for the GPU parity tests: run one case through the C-ABI and compare
it element by element with the CPU oracle.

Tolerances (the acceptance bar of this repository):
  * relative Frobenius error  ||C - ref||_F / ||ref||_F <= 1e-3
  * every element             |C - ref| <= 1e-2 * max(1, |ref|)
and a sanity band well below them: fp32 accumulation of K exact bf16 products
has a relative Frobenius error near sqrt(K) * 2^-24, so anything above 1e-4
means a narrowed accumulator or operand, not rounding noise.
"""
from __future__ import annotations

import numpy as np

REL_FRO_TOL = 1e-3
ELEM_TOL = 1e-2
SANITY_FRO = 1e-4            # fp32 output: accumulation noise is a few 1e-6, 1e-5 with a GELU
# bf16 output: both sides round an fp32 value to bf16, and where the two fp32 values lie on either side of
# a rounding boundary the results differ by one bf16 ulp (3.9e-3 relative).  A fraction f of such elements
# gives a Frobenius error of about sqrt(f) * 2.3e-3 (an ulp error averaged over the mantissa); f is the
# fp32 error over the bf16 spacing, up to about 1e-5 / 3.9e-3 = 0.3 %, i.e. 1.2e-4: the band is 5e-4.
SANITY_FRO_BF16_OUT = 5e-4
CANARY = -7.0e30


def torch_device():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch.device("cuda:0")


def to_device(x):
    """numpy -> device tensor; uint16 bf16 bit patterns travel as int16."""
    import torch
    if x is None:
        return None
    if x.dtype == np.uint16:
        return torch.from_numpy(x.view(np.int16).copy()).to(torch_device())
    return torch.from_numpy(np.ascontiguousarray(x)).to(torch_device())


def compare(got: np.ndarray, ref: np.ndarray, what: str = "", bf16_out: bool = False):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    diff = np.abs(got - ref)
    bound = ELEM_TOL * np.maximum(1.0, np.abs(ref))
    worst = int(np.argmax(diff - bound))
    assert np.all(diff <= bound), (
        f"{what}: element {np.unravel_index(worst, ref.shape)} got {got.flat[worst]!r} "
        f"ref {ref.flat[worst]!r}")
    nref = np.linalg.norm(ref)
    nerr = np.linalg.norm(got - ref)
    if nref == 0.0:
        assert np.linalg.norm(got) == 0.0, f"{what}: reference is zero, output is not"
        return 0.0
    rel = nerr / nref
    assert rel <= REL_FRO_TOL, f"{what}: relative Frobenius error {rel:.3e}"
    band = SANITY_FRO_BF16_OUT if bf16_out else SANITY_FRO
    assert rel <= band, f"{what}: error {rel:.3e} is far above fp32 accumulation noise"
    return rel


def run_case(oracle, dtype, M, N, K, *, batch=1, alpha=1.0, act="none", with_bias=True,
             lda=None, ldb=None, ldc=None, seed=0, misalign=0, plan=None, split_k=0,
             workspace="library", dist="uniform", rows=None):
    """Run the HIP path and the oracle on the same seeded inputs.

    Leading dimensions default to packed.  ``misalign`` shifts every device
    pointer by that many elements (forces the guarded kernels).  Padding of A
    and B holds large finite garbage, padding of C a canary that must survive.
    Returns (got, ref, relative Frobenius error).
    """
    import torch
    from paper_2604_01489_amd import binding, inputs as gen

    lda = K if lda is None else lda
    ldb = N if ldb is None else ldb
    ldc = N if ldc is None else ldc
    rng = np.random.default_rng(1000 + seed)

    def draw(stream, n):
        if dist == "uniform":
            return gen.uniform(seed, stream, n, -1.0, 1.0)
        return gen.normal(seed, stream, n, 1.0)

    A = draw(gen.STREAM_A, batch * M * K).reshape(batch, M, K)
    B = draw(gen.STREAM_B, batch * K * N).reshape(batch, K, N)
    bias = gen.uniform(seed, gen.STREAM_BIAS, N, -1.0, 1.0) if with_bias else None
    if dtype == "bf16":
        A, B = gen.to_bf16_bits(A), gen.to_bf16_bits(B)
        junk = np.uint16(0x7F00)          # 1.7e38: finite garbage in the padding
    else:
        junk = np.float32(3.0e37)
    Ap = np.full((batch, M, lda), junk, dtype=A.dtype); Ap[:, :, :K] = A
    Bp = np.full((batch, K, ldb), junk, dtype=B.dtype); Bp[:, :, :N] = B

    def shifted(flat):
        buf = np.full(flat.size + misalign, junk, dtype=flat.dtype)
        buf[misalign:] = flat
        t = to_device(buf)
        return t, t[misalign:]

    keepA, dA = shifted(Ap.ravel())
    keepB, dB = shifted(Bp.ravel())
    dbias = to_device(bias)
    Cbuf = torch.full((batch * M * ldc + misalign,), CANARY, dtype=torch.float32, device=torch_device())
    dC = Cbuf[misalign:]
    torch.cuda.synchronize()
    print(f"case {dtype} M={M} N={N} K={K} batch={batch} lda={lda} ldb={ldb} ldc={ldc} act={act} "
          f"bias={with_bias} alpha={alpha} misalign={misalign} plan={plan} split_k={split_k}", flush=True)
    if dtype == "bf16":
        if plan is None:
            binding.gemm_epilogue_bf16(M, N, K, dA, lda, dB, ldb, dbias, alpha, act, dC, ldc, batch)
        else:
            ws = None
            if workspace == "caller":
                nbytes = binding.workspace_bytes(M, N, K, batch, plan, split_k)
                ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device=torch_device())
            binding.gemm_epilogue_bf16_ex(M, N, K, dA, lda, dB, ldb, dbias, alpha, act, dC, ldc, batch,
                                          plan=plan, split_k=split_k, workspace=ws)
    else:
        binding.gemm_epilogue_f32(M, N, K, dA, lda, dB, ldb, dbias, alpha, act, dC, ldc, batch)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    out = Cbuf.cpu().numpy()
    assert np.all(out[:misalign] == np.float32(CANARY)), "wrote before C"
    Cp = out[misalign:].reshape(batch, M, ldc)
    assert np.all(Cp[:, :, N:] == np.float32(CANARY)), f"{cfg}: wrote into the padding of C"
    got = Cp[:, :, :N]
    ref = oracle.gemm_epilogue(A, B, bias, alpha, act)
    rel = compare(got, ref, f"{cfg} {dtype} {M}x{N}x{K}x{batch}")
    del keepA, keepB
    return got, ref, rel, cfg


def run_fused_case(oracle, M, N, K, *, batch=1, transA=False, transB=False, alpha=1.0, with_row_scale=False,
                   with_bias=True, residual=None, beta=1.0, act="none", clamp=None, out="f32",
                   pad=(0, 0, 0, 0), seed=0, misalign=0, plan="auto", split_k=0, dist="uniform",
                   a_structure="general", hint=True):
    """The widened operator through the C-ABI against its oracle on the same seeded inputs.

    ``pad`` = extra elements on (lda, ldb, ldr, ldc).  ``residual`` is None, "f32" or "bf16".
    ``misalign`` shifts the A, B and C pointers by that many elements (guarded kernel).  Padding
    of the inputs holds large finite garbage, padding of C a canary that must survive.
    ``a_structure`` "lower" / "upper" zeroes the other triangle of A (for the oracle too, which knows
    nothing of the hint) and, with ``hint``, passes the promise to the library.
    Returns (got, ref, relative Frobenius error, configuration name).
    """
    import torch
    from paper_2604_01489_amd import binding, inputs as gen

    rowsA, colsA = (K, M) if transA else (M, K)
    rowsB, colsB = (N, K) if transB else (K, N)
    lda, ldb, ldr, ldc = colsA + pad[0], colsB + pad[1], N + pad[2], N + pad[3]

    def draw(stream, n):
        if dist == "uniform":
            return gen.uniform(seed, stream, n, -1.0, 1.0)
        return gen.normal(seed, stream, n, 1.0)

    A = gen.to_bf16_bits(draw(gen.STREAM_A, batch * M * K).reshape(batch, M, K))
    if a_structure == "lower":
        A = np.tril(A)                  # applied to the last two axes: A[b, m, k] = 0 for k > m
    elif a_structure == "upper":
        A = np.triu(A)
    B = gen.to_bf16_bits(draw(gen.STREAM_B, batch * K * N).reshape(batch, K, N))
    bias = gen.uniform(seed, gen.STREAM_BIAS, N, -1.0, 1.0) if with_bias else None
    rs = gen.uniform(seed, 7, M, 0.25, 2.0) if with_row_scale else None
    junk = np.uint16(0x7F00)
    As = np.full((batch, rowsA, lda), junk, dtype=np.uint16)
    As[:, :, :colsA] = A.transpose(0, 2, 1) if transA else A
    Bs = np.full((batch, rowsB, ldb), junk, dtype=np.uint16)
    Bs[:, :, :colsB] = B.transpose(0, 2, 1) if transB else B
    Rs = None
    if residual is not None:
        R32 = gen.uniform(seed, 8, batch * M * N, -1.0, 1.0).reshape(batch, M, N)
        if residual == "bf16":
            Rs = np.full((batch, M, ldr), junk, dtype=np.uint16)
            Rs[:, :, :N] = gen.to_bf16_bits(R32)
        else:
            Rs = np.full((batch, M, ldr), np.float32(3.0e37), dtype=np.float32)
            Rs[:, :, :N] = R32

    def shifted(flat, junk_value):
        buf = np.full(flat.size + misalign, junk_value, dtype=flat.dtype)
        buf[misalign:] = flat
        t = to_device(buf)
        return t, t[misalign:]

    keepA, dA = shifted(As.ravel(), junk)
    keepB, dB = shifted(Bs.ravel(), junk)
    dbias, drs, dR = to_device(bias), to_device(rs), to_device(None if Rs is None else Rs.ravel())
    cdtype = torch.float32 if out == "f32" else torch.bfloat16
    canary = CANARY if out == "f32" else -7.0e30
    Cbuf = torch.full((batch * M * ldc + misalign,), canary, dtype=cdtype, device=torch_device())
    dC = Cbuf[misalign:]
    if dR is not None and residual == "bf16":
        dR = dR.view(torch.bfloat16)
    torch.cuda.synchronize()
    print(f"fused case M={M} N={N} K={K} batch={batch} tA={transA} tB={transB} pad={pad} act={act} out={out} "
          f"res={residual} rs={with_row_scale} bias={with_bias} clamp={clamp} misalign={misalign} plan={plan} "
          f"split_k={split_k}", flush=True)
    binding.gemm_epilogue_bf16_fused(M, N, K, dA, lda, dB, ldb, dC, ldc, batch=batch, transA=transA, transB=transB,
                                     alpha=alpha, row_scale=drs, bias=dbias, residual=dR, ldr=ldr, beta=beta,
                                     act=act, clamp=clamp, plan=plan, split_k=split_k,
                                     a_structure=a_structure if hint else "general")
    torch.cuda.synchronize()
    cfg = binding.last_config()
    outv = Cbuf.to(torch.float32).cpu().numpy()
    canary32 = np.float32(torch.tensor(canary, dtype=cdtype).to(torch.float32).item())
    assert np.all(outv[:misalign] == canary32), "wrote before C"
    Cp = outv[misalign:].reshape(batch, M, ldc)
    assert np.all(Cp[:, :, N:] == canary32), f"{cfg}: wrote into the padding of C"
    got = Cp[:, :, :N]
    ref = oracle.gemm_fused(M, N, K, As, Bs, batch=batch, transA=transA, transB=transB, lda=lda, ldb=ldb,
                            alpha=alpha, row_scale=rs, bias=bias, residual=Rs, ldr=ldr, beta=beta, act=act,
                            clamp=clamp, out=out)
    rel = compare(got, ref, f"{cfg} fused {M}x{N}x{K}x{batch}", bf16_out=(out == "bf16"))
    del keepA, keepB
    return got, ref, rel, cfg
