"""The entry points enqueue kernels only (no allocation, no memset, no synchronisation when the
caller provides the split-K workspace), so a stream capture of them replays correctly.  Every
replay is checked against the eager result, with eager work and synchronisations between replays."""
import numpy as np
import pytest

from paper_2604_01489_amd import binding

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("force", [None, "256x256"])
def test_calls_replay_from_a_captured_graph(force, monkeypatch):
    """As the planner routes them (128 x 128 tiles at these sizes) and with the 256 x 256 tile forced, which
    puts all three calls on the four-wave kernel (plain, partial tiles, bf16 output through LDS)."""
    import torch
    from paper_2604_01489_amd import inputs as gen
    if force:
        binding.set_option("force_config", force)
    dev = torch.device("cuda:0")
    M, N, K = 512, 512, 256
    A = torch.from_numpy(gen.to_bf16_bits(gen.normal(70, 0, M * K, K ** -0.5).reshape(M, K)).view(np.int16)).to(dev)
    B = torch.from_numpy(gen.to_bf16_bits(gen.normal(70, 1, K * N, 1.0).reshape(K, N)).view(np.int16)).to(dev)
    bias = torch.from_numpy(gen.uniform(70, 2, N, -1.0, 1.0)).to(dev)
    Kbig = 8192
    A2 = torch.from_numpy(gen.to_bf16_bits(gen.normal(71, 0, 256 * Kbig, Kbig ** -0.5).reshape(256, Kbig)).view(np.int16)).to(dev)
    B2 = torch.from_numpy(gen.to_bf16_bits(gen.normal(71, 1, Kbig * 256, 1.0).reshape(Kbig, 256)).view(np.int16)).to(dev)
    split = 8
    ws = torch.empty(binding.workspace_bytes(256, 256, Kbig, 1, "splitk", split) // 4, dtype=torch.float32, device=dev)

    def enqueue(C1, C2, C3, stream):
        binding.gemm_epilogue_bf16(M, N, K, A, K, B, N, bias, 0.5, "gelu_tanh", C1, N, stream=stream)
        binding.gemm_epilogue_bf16_ex(256, 256, Kbig, A2, Kbig, B2, 256, None, 1.0, "none", C2, 256, plan="splitk",
                                      split_k=split, workspace=ws, stream=stream)
        binding.gemm_epilogue_bf16_fused(M, N, K, A, K, B, N, C3, N, alpha=0.5, bias=bias, act="relu", clamp=(0.0, 1.0),
                                         stream=stream)

    eager = [torch.empty(M, N, device=dev), torch.empty(256, 256, device=dev), torch.empty(M, N, dtype=torch.bfloat16, device=dev)]
    enqueue(*eager, torch.cuda.current_stream())
    torch.cuda.synchronize()
    if force:
        assert binding.last_config() == "bf16_fused_256x256x64_w4_nn", binding.last_config()

    out = [torch.zeros_like(t) for t in eager]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        print("capturing", flush=True)
        with torch.cuda.graph(graph, stream=side):
            enqueue(*out, torch.cuda.current_stream())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in out:
            t.fill_(-1.0)                    # eager work between replays
        torch.cuda.synchronize()
        print(f"replay {replay}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(out, eager):
            assert torch.equal(got, want), f"replay {replay} differs from the eager result"


def test_convolution_rowsum_and_structured_calls_replay_from_a_captured_graph():
    """The convolution (gathering kernel and few-channel kernel), the row-sum pair (weights stored K x N: no
    workspace), the diagonal operand, a product with a promised triangular A, a tall product with 8 columns and a
    symmetric operand with the caller's workspace: kernels only, so their capture replays bit for bit."""
    import torch
    from paper_2604_01489_amd import inputs as gen
    dev = torch.device("cuda:0")

    def bf16(seed, stream, shape, scale=1.0):
        return torch.from_numpy(gen.to_bf16_bits(gen.normal(seed, stream, int(np.prod(shape)), scale).reshape(shape))
                                .view(np.int16)).to(dev)

    X, Wt = bf16(80, 0, (2, 20, 20, 64)), bf16(80, 1, (72, 3, 3, 64), 576 ** -0.5)
    M, N, K = 520, 264, 520
    A = torch.from_numpy(np.tril(gen.to_bf16_bits(gen.normal(81, 0, M * K, K ** -0.5).reshape(M, K))).view(np.int16)).to(dev)
    B = bf16(81, 1, (K, N))
    bias = torch.from_numpy(gen.uniform(81, 2, N, -1.0, 1.0)).to(dev)
    d = torch.from_numpy(gen.uniform(82, 7, K, 0.5, 1.5)).to(dev)
    X3, W3 = bf16(83, 0, (2, 30, 38, 3)), bf16(83, 1, (64, 7, 7, 3), 147 ** -0.5)
    Mt, Nt, Kt = 2080, 8, 520
    At, Bt = bf16(84, 0, (Mt, Kt), Kt ** -0.5), bf16(84, 1, (Kt, Nt))
    Ms, Ns = 768, 16
    As, Bs = bf16(85, 0, (Ms, Ms), Ms ** -0.5), bf16(85, 1, (Ms, Ns))
    sym_args = binding.fused_args(Ms, Ns, Ms, As.data_ptr(), Ms, Bs.data_ptr(), Ns, As.data_ptr(), Ns, a_structure="sym_lower")      # sizes and alignment only
    ws = torch.empty(max(binding.fused_workspace_bytes(sym_args) // 4, 1), dtype=torch.float32, device=dev)

    def enqueue(Y, C, params, y, D, Y3, Ct, Cs, stream):
        binding.conv2d_epilogue_bf16(X, Wt, Y, pad=(1, 1), act="relu", stream=stream)
        binding.gemm_epilogue_bf16_fused(M, N, K, A, K, B, N, C, N, bias=bias, act="relu", a_structure="lower", stream=stream)
        binding.gemm_rowsum_params_bf16(N, K, B, N, False, bias, params, stream=stream)
        binding.gemm_rowsum_bf16(M, K, A, K, params, 0.5, y, stream=stream)
        binding.gemm_epilogue_diag_bf16(K, N, d, B, N, bias, 0.5, "relu", D, N, 1, stream=stream)
        binding.conv2d_epilogue_bf16(X3, W3, Y3, stride=(2, 2), pad=(3, 3), act="relu", stream=stream)
        assert binding.last_config() == "conv_bf16_rows_k32"
        binding.gemm_epilogue_bf16(Mt, Nt, Kt, At, Kt, Bt, Nt, None, 0.5, "gelu_tanh", Ct, Nt, stream=stream)
        assert binding.last_config().startswith("bf16_skinny")
        binding.gemm_epilogue_bf16_fused(Ms, Ns, Ms, As, Ms, Bs, Ns, Cs, Ns, act="relu", a_structure="sym_lower", workspace=ws,
                                         stream=stream)
        assert binding.last_config().startswith("bf16_symm_lower")

    def buffers():
        return [torch.empty(2, 20, 20, 72, dtype=torch.bfloat16, device=dev), torch.empty(M, N, device=dev),
                torch.empty(K + 1, device=dev), torch.empty(M, device=dev), torch.empty(K, N, device=dev),
                torch.empty(2, 15, 19, 64, dtype=torch.bfloat16, device=dev), torch.empty(Mt, Nt, device=dev),
                torch.empty(Ms, Ns, device=dev)]

    eager = buffers()
    enqueue(*eager, torch.cuda.current_stream())
    torch.cuda.synchronize()
    out = buffers()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        print("capturing", flush=True)
        with torch.cuda.graph(graph, stream=side):
            enqueue(*out, torch.cuda.current_stream())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for replay in range(3):
        for t in out:
            t.fill_(-1.0)
        torch.cuda.synchronize()
        print(f"replay {replay}", flush=True)
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip(out, eager):
            assert torch.equal(got, want), f"replay {replay} differs from the eager result"
