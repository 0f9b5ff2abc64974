"""The synthetic workloads at full size, in the launch configuration bench.py
times (plain gemm_epilogue_* calls, library-chosen plan), checked against the oracle
on sampled rows of C (whole first and last tiles' rows included) -- the oracle computes
each sampled row exactly as it would in a full run.  The small fp32 workload is compared
in full."""
import numpy as np
import pytest

from gpu_util import compare, to_device

pytestmark = pytest.mark.gpu


def _sample_rows(M, count):
    """Blocks of 32 rows spread over M, first and last block included, not tile aligned."""
    if count >= M:
        return np.arange(M)
    blocks = max(2, count // 32)
    starts = np.unique(np.round(np.linspace(0, M - 32, blocks)).astype(np.int64))
    starts = np.clip(starts + (np.arange(starts.size) % 5) * 3, 0, M - 32)
    starts[0], starts[-1] = 0, M - 32
    return np.unique((starts[:, None] + np.arange(32)[None, :]).ravel())


def _run_workload(oracle, name, rows_wanted, batches_wanted=4):
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    w = gen.WORKLOADS[name]
    A, B, bias = gen.make_inputs(w)
    dA, dB, dbias = to_device(A), to_device(B), to_device(bias)
    C = torch.empty(w.batch, w.M, w.N, dtype=torch.float32, device="cuda:0")
    print(f"workload {name}", flush=True)
    call = binding.gemm_epilogue_bf16 if w.dtype == "bf16" else binding.gemm_epilogue_f32
    call(w.M, w.N, w.K, dA, w.K, dB, w.N, dbias, w.alpha, w.act, C, w.N, w.batch)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    rows = _sample_rows(w.M, rows_wanted)
    bsel = np.unique(np.round(np.linspace(0, w.batch - 1, min(w.batch, batches_wanted))).astype(np.int64))
    got = C[torch.from_numpy(bsel).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy()
    ref = oracle.gemm_epilogue(np.ascontiguousarray(A[bsel][:, rows]), np.ascontiguousarray(B[bsel]),
                               bias, w.alpha, w.act)
    rel = compare(got, ref, f"{name} [{cfg}]")
    return C, cfg, rel


def test_c1_f32_256_full(oracle):
    _, cfg, _ = _run_workload(oracle, "c1_f32_256", 256)
    assert cfg.startswith("f32_")


def test_c2_bf16_4096(oracle):
    _, cfg, _ = _run_workload(oracle, "c2_bf16_4096", 320)
    assert cfg == "bf16_256x256x64_w4"


def test_c3_bf16_8192_bias_gelu(oracle):
    _, cfg, _ = _run_workload(oracle, "c3_bf16_8192_bias_gelu", 320)
    assert cfg == "bf16_256x256x64_w4"


def test_c4_bf16_batched(oracle):
    C, cfg, _ = _run_workload(oracle, "c4_bf16_batched_512x512x64", 512, batches_wanted=6)
    assert cfg.startswith("bf16_")
    # relu output: no negative value anywhere in the full result
    assert float(C.min()) >= 0.0


def test_c5_bf16_splitk(oracle):
    import torch
    C1, cfg, _ = _run_workload(oracle, "c5_bf16_splitk_1024x1024x65536", 160)
    assert cfg.endswith("_splitk")
    C2, _, _ = _run_workload(oracle, "c5_bf16_splitk_1024x1024x65536", 32)
    assert torch.equal(C1, C2), "split-K result must be bitwise repeatable"


# ---------------------------------------------------------------- the widened operator's workloads
def _run_fused_workload(oracle, name, rows_wanted, batches_wanted=4, cross_check=False):
    """Full-size fused workload through gemm_epilogue_bf16_fused, sampled rows against its oracle
    (a row of the sample is computed exactly as in a full run: the oracle has one k loop per output)."""
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    fw = gen.FUSED_WORKLOADS[name]
    w = fw.base
    host = gen.make_fused_inputs(fw)
    A, B = host["A"], host["B"]
    dA, dB, dbias = to_device(A), to_device(B), to_device(host["bias"])
    drs, dR = to_device(host["row_scale"]), to_device(host["residual"])
    if dR is not None and fw.residual == "bf16":
        dR = dR.view(torch.bfloat16)
    C = torch.empty(w.batch, w.M, w.N, dtype=torch.float32 if fw.out == "f32" else torch.bfloat16, device="cuda:0")
    print(f"fused workload {name}", flush=True)
    binding.gemm_epilogue_bf16_fused(w.M, w.N, w.K, dA, A.shape[2], dB, B.shape[2], C, w.N, batch=w.batch,
                                     transA=fw.transA, transB=fw.transB, alpha=w.alpha, row_scale=drs, bias=dbias,
                                     residual=dR, ldr=w.N, beta=fw.beta, act=w.act, clamp=fw.clamp,
                                     a_structure=fw.a_structure)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    rows = _sample_rows(w.M, rows_wanted)
    bsel = np.unique(np.round(np.linspace(0, w.batch - 1, min(w.batch, batches_wanted))).astype(np.int64))
    got = C[torch.from_numpy(bsel).cuda()][:, torch.from_numpy(rows).cuda()].to(torch.float32).cpu().numpy()
    A_s = np.ascontiguousarray(A[bsel][:, :, rows] if fw.transA else A[bsel][:, rows])
    rs_s = None if host["row_scale"] is None else host["row_scale"][rows]
    R_s = None if host["residual"] is None else np.ascontiguousarray(host["residual"][bsel][:, rows])
    ref = oracle.gemm_fused(len(rows), w.N, w.K, A_s, np.ascontiguousarray(B[bsel]), batch=len(bsel),
                            transA=fw.transA, transB=fw.transB, alpha=w.alpha, row_scale=rs_s, bias=host["bias"],
                            residual=R_s, beta=fw.beta, act=w.act, clamp=fw.clamp, out=fw.out)
    compare(got, ref, f"{name} [{cfg}]", bf16_out=(fw.out == "bf16"))
    if cross_check:
        # Every element, not only the sampled rows: the same call through the guarded kernel (parity-tested
        # against the oracle on its own), compared on the device to the elementwise bound of the tolerance.
        binding.set_option("force_config", "generic")
        C2 = torch.empty_like(C)
        binding.gemm_epilogue_bf16_fused(w.M, w.N, w.K, dA, A.shape[2], dB, B.shape[2], C2, w.N, batch=w.batch,
                                         transA=fw.transA, transB=fw.transB, alpha=w.alpha, row_scale=drs, bias=dbias,
                                         residual=dR, ldr=w.N, beta=fw.beta, act=w.act, clamp=fw.clamp,
                                         a_structure=fw.a_structure)
        torch.cuda.synchronize()
        binding.set_option("force_config", None)
        assert "generic" in binding.last_config(), binding.last_config()
        a, b = C.float(), C2.float()
        bad = (a - b).abs() > 1e-2 * torch.clamp(b.abs(), min=1.0)
        assert not bool(bad.any()), f"{name}: {int(bad.sum())} elements differ between {cfg} and the guarded kernel"
    return C, cfg


def test_c6_fused_nt_bf16out(oracle):
    _, cfg = _run_fused_workload(oracle, "c6_fused_nt_8192_bias_gelu_bf16out", 160, cross_check=True)
    assert cfg == "bf16_fused_256x256x64_w4_nt"


def test_c7_fused_tn_chain(oracle):
    C, cfg = _run_fused_workload(oracle, "c7_fused_tn_8192_chain", 160, cross_check=True)
    assert cfg == "bf16_fused_256x256x32_w8_tn"
    assert 0.0 <= float(C.float().min()) and float(C.float().max()) <= 6.0      # relu then clamp(0, 6), everywhere


def test_c8_fused_batched_bf16out(oracle):
    C, cfg = _run_fused_workload(oracle, "c8_fused_batched_512x512x64_bf16out", 512, batches_wanted=6)
    assert cfg in ("bf16_fused_256x256x32_w8_nn", "bf16_fused_128x128x32_w4_nn")      # the planner's measured per-round costs decide
    assert float(C.float().min()) >= 0.0


# ---------------------------------------------------------------- structured operand and convolution
def test_c9_diag_full(oracle):
    """C = relu(alpha diag(d) B + bias) at 8192^2: every row of a sample against the operator's definition
    with the dense matrix diag(d) as A (the fused oracle with A = I and row scale d)."""
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    w = gen.DIAG_WORKLOADS["c9_diag_bf16_8192"]
    d, B, bias = gen.make_diag_inputs(w)
    dd, dB, dbias = to_device(d), to_device(B), to_device(bias)
    C = torch.empty(w.batch, w.M, w.N, dtype=torch.float32, device="cuda:0")
    print("workload c9_diag_bf16_8192", flush=True)
    binding.gemm_epilogue_diag_bf16(w.M, w.N, dd, dB, w.N, dbias, w.alpha, w.act, C, w.N, w.batch)
    torch.cuda.synchronize()
    assert binding.last_config() == "diag_rows_vec4"
    rows = _sample_rows(w.M, 256)
    got = C[:, torch.from_numpy(rows).cuda()].cpu().numpy()
    # row m of diag(d) B is d[m] times row m of B: as a GEMM over the sampled rows, A = I (K = rows), scaled per row
    eye = gen.to_bf16_bits(np.eye(len(rows), dtype=np.float64))[None]
    ref = oracle.gemm_fused(len(rows), w.N, len(rows), eye, np.ascontiguousarray(B[:, rows]), batch=w.batch,
                            alpha=w.alpha, row_scale=d[rows], bias=bias, act=w.act, out="f32")
    compare(got, ref, "c9_diag_bf16_8192 [diag_rows_vec4]")


def _run_conv_workload(oracle, name, expect, imgs):
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    cw = gen.CONV_WORKLOADS[name]
    host = gen.make_conv_inputs(cw)
    oh, ow = cw.out_hw()
    dX, dW, dbias, dR = to_device(host["X"]), to_device(host["Wt"]), to_device(host["bias"]), to_device(host["residual"])
    if dR is not None and cw.residual == "bf16":
        dR = dR.view(torch.bfloat16)
    Y = torch.empty(cw.N, oh, ow, cw.Cout, dtype=torch.float32 if cw.out == "f32" else torch.bfloat16, device="cuda:0")
    print(f"workload {name}", flush=True)
    binding.conv2d_epilogue_bf16(dX, dW, Y, stride=cw.stride, pad=cw.pad, dil=cw.dil, alpha=cw.alpha, bias=dbias,
                                 residual=dR, beta=cw.beta, act=cw.act, clamp=cw.clamp)
    torch.cuda.synchronize()
    cfg = binding.last_config()
    assert cfg == expect
    sub = gen.make_conv_inputs(cw, imgs)
    got = Y[torch.tensor(imgs, device="cuda:0")].to(torch.float32).cpu().numpy()
    ref = oracle.conv2d_nhwc(sub["X"], sub["Wt"], stride=cw.stride, pad=cw.pad, dil=cw.dil, alpha=cw.alpha,
                             bias=sub["bias"], residual=sub["residual"], beta=cw.beta, act=cw.act, clamp=cw.clamp,
                             out=cw.out)
    compare(got.reshape(1, -1, cw.Cout), ref.reshape(1, -1, cw.Cout), f"{name} [{cfg}]", bf16_out=(cw.out == "bf16"))
    return Y, cw


def test_c10_conv_full(oracle):
    """The 3x3 convolution workload at full size: first and last image (first and last tiles of the implicit
    GEMM) and one in the middle against the convolution oracle, every position and channel: on the halo-staged
    kernel, which the plan picks (tiles of 4 and of 3 output rows, one of each per CU), and on the gathering kernel;
    the two outputs also against each other over all images."""
    import torch
    from paper_2604_01489_amd import binding
    Yh, _ = _run_conv_workload(oracle, "c10_conv3x3_256_bf16out", "conv_bf16_halo_3x3_w4_14_11", [0, 13, 31])
    binding.set_option("conv_halo", "off")
    Yg, _ = _run_conv_workload(oracle, "c10_conv3x3_256_bf16out", "conv_bf16_256x256x32_w8", [0, 31])
    # same products, summed in a different order, rounded to bf16: within two units in the last place of each other
    diff = (Yh.to(torch.float32) - Yg.to(torch.float32)).abs()
    assert bool((diff <= 2.0 ** -7 * torch.maximum(Yg.to(torch.float32).abs(), torch.tensor(2.0 ** -3, device="cuda:0"))).all())


def test_c15_conv_first_layer_full(oracle):
    """The first-layer workload (3 channels, 7 x 7, stride 2) at full size: the first, a middle and the last image
    against the convolution oracle, every position and channel; relu output, so nothing negative anywhere."""
    Y, _ = _run_conv_workload(oracle, "c15_conv7x7_first_layer_bf16out", "conv_bf16_rows_k32", [0, 13, 31])
    assert float(Y.float().min()) >= 0.0


def test_c11_fused_lower_triangular(oracle):
    """8192^3 with a lower-triangular A and the caller's promise: sampled rows (first and last tile
    rows included: the shortest and the longest K range) against the oracle, which is told nothing."""
    _, cfg = _run_fused_workload(oracle, "c11_fused_lower_8192_bias_relu", 160, cross_check=True)
    assert cfg == "bf16_fused_256x256x64_w4_nn"


def test_c12_rowsum_linear_full(oracle):
    """The row sum of an 8192 x 8192 linear layer over 8192 inputs by the collapsed form: sampled rows
    against the definition (full product in fp64, then the sum over the output dimension)."""
    import torch
    from paper_2604_01489_amd import binding, inputs as gen
    w = gen.ROWSUM_WORKLOADS["c12_rowsum_linear_8192"]
    A, Wt, bias = gen.make_rowsum_inputs(w)
    dA, dW, dbias = to_device(A), to_device(Wt), to_device(bias)
    params = torch.empty(w.K + 1, dtype=torch.float32, device="cuda:0")
    y = torch.empty(w.M, dtype=torch.float32, device="cuda:0")
    print("workload c12_rowsum_linear_8192", flush=True)
    binding.gemm_rowsum_params_bf16(w.N, w.K, dW, w.K, True, dbias, params)
    assert binding.last_config() == "rowsum_params_cols"
    binding.gemm_rowsum_bf16(w.M, w.K, dA, w.K, params, w.alpha, y)
    assert binding.last_config() == "rowsum_rows_wide"
    torch.cuda.synchronize()
    rows = _sample_rows(w.M, 128)
    got = y[torch.from_numpy(rows).cuda()].cpu().numpy()[None, :, None]
    ref = oracle.gemm_rowsum(np.ascontiguousarray(A[rows]), np.ascontiguousarray(Wt.T), bias, w.alpha)[None, :, None]
    compare(got, ref, "c12_rowsum_linear_8192 [rowsum_rows_wide]")
