"""Host-side checks that need no GPU: the library loads, exports every symbol the
header declares, validates arguments before touching a device and plans split-K
as documented."""
import os
import re

import pytest

from paper_2604_01489_amd import binding, build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not build.library_is_current():
        build.build_library()
    return binding.load()


def declared_in(header_file):
    text = open(os.path.join(ROOT, "include", header_file)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(ge_\w+|gemm_epilogue\w*|conv2d_epilogue\w*|gemm_rowsum\w*)\s*\(", text))


def test_exports_every_declared_symbol(lib):
    """Each header against the library that implements it: the operator, and the measurement probes."""
    assert sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")) == ["ge_probes.h", "gemm_epilogue.h"]
    declared = declared_in("gemm_epilogue.h")
    assert declared == set(binding.SYMBOLS), declared ^ set(binding.SYMBOLS)
    for name in declared:
        assert getattr(lib, name) is not None
    probes = binding.load_probes()
    declared = declared_in("ge_probes.h")
    assert declared == set(binding.PROBE_SYMBOLS), declared ^ set(binding.PROBE_SYMBOLS)
    for name in declared:
        assert getattr(probes, name) is not None
        assert not hasattr(lib, name), f"{name} belongs to the probes library, not to the operator's"


def test_options_are_validated_and_restorable(lib):
    """ge_set_option: known names and values only; NULL restores the default."""
    assert lib.ge_set_option(None, b"8") == 1
    assert lib.ge_set_option(b"no_such_switch", b"1") == 8
    assert lib.ge_set_option(b"force_config", b"512x512") == 8
    assert lib.ge_set_option(b"waves", b"16") == 8 and lib.ge_set_option(b"stage_k", b"48") == 8
    try:
        # the switch changes the plan the host-side queries report
        assert binding.auto_split_k(2048, 2048, 2048) == 1
        binding.set_option("force_config", "256x256")
        forced = binding.auto_split_k(2048, 2048, 2048)
        binding.set_option("force_config", None)
        assert binding.auto_split_k(2048, 2048, 2048) == 1
        assert forced >= 1
        for name, value in (("force_config", "128x128"), ("force_config", "generic"), ("waves", "8"), ("waves", "4"),
                            ("stage_k", "32"), ("stage_k", "64")):
            binding.set_option(name, value)
    finally:
        for name in ("force_config", "waves", "stage_k"):
            binding.set_option(name, None)


def test_symmetric_plan_and_workspace_queries(lib):
    """Host only: a symmetric A with few output columns asks for the workspace of its partial results
    (terms x batch x M x N floats); the same call with many columns runs in the guarded kernel, one pass."""
    few = binding.fused_args(8192, 16, 8192, P, 8192, P, 16, P, 16, a_structure="sym_lower")
    assert binding.fused_workspace_bytes(few) == 32 * 8192 * 16 * 4          # 32 rows of super-tiles of 256
    big = binding.fused_args(16384, 16, 16384, P, 16384, P, 16, P, 16, a_structure="sym_upper")
    assert binding.fused_workspace_bytes(big) == 22 * 16384 * 16 * 4         # 22 rows of super-tiles of 768: one round
    many = binding.fused_args(1024, 64, 1024, P, 1024, P, 64, P, 64, a_structure="sym_lower", plan="direct")
    assert binding.fused_workspace_bytes(many) == 0
    assert binding.fused_workspace_bytes(binding.fused_args(1024, 8, 512, P, 1024, P, 8, P, 8, a_structure="sym_lower")) == 0
    # the general split-K call answers as gemm_epilogue_workspace_bytes does
    g = binding.fused_args(1024, 1024, 65536, P, 65536, P, 1024, P, 1024)
    assert binding.fused_workspace_bytes(g) == binding.workspace_bytes(1024, 1024, 65536)
    assert binding.rowsum_params_workspace_bytes(8192, 8192, True) == 128 * 8192 * 4
    assert binding.rowsum_params_workspace_bytes(8192, 8192, False) == 0


def test_conv_workspace_query(lib):
    """Host only: a late layer (few output tiles, long K) is split over K and says how many bytes its
    partial results take; an early layer runs in one pass; invalid sizes report 0."""
    late = binding.conv_args((32, 7, 7, 512, 512, 3, 3), P, P, P, pad=(1, 1), y_type="bf16")
    early = binding.conv_args((32, 56, 56, 256, 256, 3, 3), P, P, P, pad=(1, 1), y_type="bf16")
    bad = binding.conv_args((32, 7, 7, 0, 512, 3, 3), P, P, P)
    n = binding.conv_workspace_bytes(late)
    assert n > 0 and n % (32 * 7 * 7 * 512 * 4) == 0
    assert binding.conv_workspace_bytes(early) == 0 and binding.conv_workspace_bytes(bad) == 0
    # few input channels: the row kernel runs in one pass whatever the guarded kernel's planner would have sliced
    first = binding.conv_args((1, 12, 12, 3, 64, 7, 7), P, P, P, stride=(2, 2), pad=(3, 3), y_type="bf16")
    assert binding.conv_workspace_bytes(first) == 0
    # a workspace that is too small or misaligned is refused before anything is enqueued
    small = binding.conv_args((32, 7, 7, 512, 512, 3, 3), P, P, P, pad=(1, 1), y_type="bf16", workspace_ptr=P,
                              workspace_bytes=n - 1)
    assert binding.raw_conv(small) == 6
    odd = binding.conv_args((32, 7, 7, 512, 512, 3, 3), P, P, P, pad=(1, 1), y_type="bf16", workspace_ptr=P + 16,
                            workspace_bytes=n)
    assert binding.raw_conv(odd) == 6


def test_status_strings(lib):
    seen = {binding.status_string(i) for i in range(10)}
    assert len(seen) == 10 and "ok" in seen
    assert binding.status_string(99) == "unknown status"


P = 0x10000  # a plausible, suitably aligned fake device address: never dereferenced on error paths


@pytest.mark.parametrize("name", ["gemm_epilogue_bf16", "gemm_epilogue_f32"])
def test_argument_errors_return_codes(lib, name):
    call = lambda *a: binding.raw_call(name, *a)
    ok = (64, 64, 64, P, 64, P, 64, None, 1.0, 0, P, 64, 1)

    def with_(**kw):
        names = ["M", "N", "K", "A", "lda", "B", "ldb", "bias", "alpha", "act", "C", "ldc", "batch"]
        vals = list(ok)
        for k, v in kw.items():
            vals[names.index(k)] = v
        return call(*vals)

    assert with_(A=None) == 1 and with_(B=None) == 1 and with_(C=None) == 1
    assert with_(M=0) == 2 and with_(N=-1) == 2 and with_(K=0) == 2 and with_(batch=0) == 2
    assert with_(lda=63) == 3 and with_(ldb=63) == 3 and with_(ldc=63) == 3
    assert with_(act=3) == 4 and with_(act=-1) == 4
    assert with_(A=P + 1) == 5 and with_(C=P + 2) == 5 and with_(bias=P + 1) == 5
    if name.endswith("f32"):
        assert with_(B=P + 2) == 5


def test_fused_argument_errors_return_codes(lib):
    """gemm_epilogue_bf16_fused validates before it touches a device (the addresses are fake)."""
    def call(**kw):
        a = dict(M=64, N=48, K=32, A_ptr=P, lda=32, B_ptr=P, ldb=48, C_ptr=P, ldc=48)
        a.update(kw)
        pos = [a.pop(k) for k in ("M", "N", "K", "A_ptr", "lda", "B_ptr", "ldb", "C_ptr", "ldc")]
        return binding.raw_fused(binding.fused_args(*pos, **a))

    assert call(A_ptr=None) == 1 and call(B_ptr=None) == 1 and call(C_ptr=None) == 1
    assert call(M=0) == 2 and call(batch=0) == 2
    # leading dimensions follow the storage: lda >= K, or >= M when A is stored transposed
    assert call(lda=31) == 3 and call(transA=True, lda=63) == 3
    assert call(ldb=47) == 3 and call(transB=True, ldb=31) == 3
    assert call(ldc=47) == 3 and call(R_ptr=P, ldr=47) == 3
    assert call(act=3) == 4
    assert call(A_ptr=P + 1) == 5 and call(C_ptr=P + 2) == 5 and call(bias_ptr=P + 2) == 5
    assert call(R_ptr=P + 2, ldr=48, r_type="f32") == 5
    assert call(row_scale_ptr=P + 1) == 5
    assert call(clamp=(1.0, 0.5)) == 9 and call(clamp=(float("nan"), 1.0)) == 9
    assert call(c_type=2) == 9
    assert call(plan=7) == 8
    # the promise about A: a known value, and never together with K slices
    assert call(a_structure=5) == 8 and call(a_structure=-1) == 8
    assert call(a_structure="lower", plan="splitk") == 8 and call(a_structure="upper", plan="splitk", split_k=4) == 8
    # bf16 output only needs 2-byte alignment of C
    assert call(C_ptr=P + 2, c_type="bf16", plan=7) == 8
    assert binding.load().gemm_epilogue_bf16_fused(None, None) == 1


def test_diag_argument_errors_return_codes(lib):
    ok = dict(M=64, N=48, d=P, B=P, ldb=48, bias=None, alpha=1.0, act=0, C=P, ldc=48, batch=1)

    def call(**kw):
        a = dict(ok)
        a.update(kw)
        return binding.raw_diag(a["M"], a["N"], a["d"], a["B"], a["ldb"], a["bias"], a["alpha"], a["act"], a["C"],
                                a["ldc"], a["batch"])

    assert call(d=None) == 1 and call(B=None) == 1 and call(C=None) == 1
    assert call(M=0) == 2 and call(N=0) == 2 and call(batch=0) == 2
    assert call(ldb=47) == 3 and call(ldc=47) == 3
    assert call(act=5) == 4
    assert call(B=P + 1) == 5 and call(C=P + 2) == 5 and call(d=P + 2) == 5 and call(bias=P + 1) == 5


def test_rowsum_argument_errors_return_codes(lib):
    assert binding.raw_rowsum_params(48, 32, None, 48, 0, None, P) == 1 and binding.raw_rowsum_params(48, 32, P, 48, 0, None, None) == 1
    assert binding.raw_rowsum_params(0, 32, P, 48, 0, None, P) == 2 and binding.raw_rowsum_params(48, 0, P, 48, 0, None, P) == 2
    assert binding.raw_rowsum_params(48, 32, P, 47, 0, None, P) == 3          # B is K x N: ldb >= N
    assert binding.raw_rowsum_params(48, 32, P, 31, 1, None, P) == 3          # B stored N x K: ldb >= K
    assert binding.raw_rowsum_params(48, 32, P + 1, 48, 0, None, P) == 5 and binding.raw_rowsum_params(48, 32, P, 48, 0, P + 2, P) == 5
    assert binding.raw_rowsum_params(48, 32, P, 48, 0, None, P + 2) == 5
    assert binding.raw_rowsum_params(65536 * 128, 8, P, 8, 1, None, P) == 2   # more column-sum chunks than the grid carries
    assert binding.raw_rowsum(64, 32, None, 32, P, 1.0, P) == 1 and binding.raw_rowsum(64, 32, P, 32, None, 1.0, P) == 1
    assert binding.raw_rowsum(64, 32, P, 32, P, 1.0, None) == 1
    assert binding.raw_rowsum(0, 32, P, 32, P, 1.0, P) == 2 and binding.raw_rowsum(64, 32, P, 31, P, 1.0, P) == 3
    assert binding.raw_rowsum(64, 32, P + 1, 32, P, 1.0, P) == 5 and binding.raw_rowsum(64, 32, P, 32, P, 1.0, P + 2) == 5


def test_conv_argument_errors_return_codes(lib):
    def call(shape=(1, 8, 8, 32, 16, 3, 3), X=P, Wt=P, Y=P, **kw):
        return binding.raw_conv(binding.conv_args(shape, X, Wt, Y, **kw))

    assert call(X=None) == 1 and call(Wt=None) == 1 and call(Y=None) == 1
    assert binding.load().conv2d_epilogue_bf16(None, None) == 1
    assert call(shape=(0, 8, 8, 32, 16, 3, 3)) == 2 and call(shape=(1, 8, 8, 0, 16, 3, 3)) == 2
    assert call(shape=(1, 2, 2, 32, 16, 3, 3)) == 2                 # kernel larger than the input: empty output
    assert call(shape=(1, 2, 2, 32, 16, 3, 3), pad=(1, 1)) == 7     # with padding it fits (no device here: launch fails)
    assert call(stride=(0, 1)) == 2 and call(pad=(-1, 0)) == 2 and call(dil=(1, 0)) == 2
    assert call(act=3) == 4
    assert call(clamp=(2.0, 1.0)) == 9 and call(y_type=2) == 9
    assert call(X=P + 1) == 5 and call(Y=P + 2) == 5 and call(bias_ptr=P + 1) == 5 and call(R_ptr=P + 2) == 5


def test_ex_plan_errors(lib):
    base = (64, 64, 64, P, 64, P, 64, None, 1.0, 0, P, 64, 1)
    assert binding.raw_call("gemm_epilogue_bf16_ex", *base, extra=(7, 0, None, 0)) == 8
    assert binding.raw_call("gemm_epilogue_bf16_ex", *base, extra=(2, -1, None, 0)) == 8
    # caller workspace too small / misaligned for a forced split
    big = (256, 256, 4096, P, 4096, P, 256, None, 1.0, 0, P, 256, 1)
    need = binding.workspace_bytes(256, 256, 4096, 1, "splitk", 4)
    assert need == 4 * 256 * 256 * 4
    assert binding.raw_call("gemm_epilogue_bf16_ex", *big, extra=(2, 4, P, need - 1)) == 6
    assert binding.raw_call("gemm_epilogue_bf16_ex", *big, extra=(2, 4, P + 16, need)) == 6


def test_split_k_planning(lib):
    # many output tiles: never split
    assert binding.auto_split_k(8192, 8192, 8192) == 1
    assert binding.auto_split_k(4096, 4096, 4096) == 1
    assert binding.auto_split_k(512, 512, 64, 256) == 1
    # 16 tiles of 256x256, K = 65536: one slice per CU
    assert binding.auto_split_k(1024, 1024, 65536) == 16
    assert binding.workspace_bytes(1024, 1024, 65536) == 16 * 1024 * 1024 * 4
    # short K is not worth slicing
    assert binding.auto_split_k(128, 128, 512) == 1
    assert binding.workspace_bytes(8192, 8192, 8192) == 0
    # forced split rounds slices to whole K tiles and drops empty ones: 5 wanted, K = 128
    # gives 2 slices of 64 with the fast kernels and 4 of 32 with the guarded one; the
    # query does not know the pointers' alignment and reports the larger need
    assert binding.workspace_bytes(256, 256, 128, 1, "splitk", 5) == 4 * 256 * 256 * 4


def test_public_headers_compile_as_plain_c(tmp_path):
    """The boundary is a C ABI: both headers are valid C99 on their own (no C++ in them, every type declared
    before use)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "hdr.c"
    src.write_text('#include "include/gemm_epilogue.h"\n#include "include/ge_probes.h"\n'
                   "int main(void) { ge_fused_args_t a; ge_conv_args_t c; a.a_structure = GE_A_LOWER; c.N = 1;\n"
                   "  return (int)(sizeof a + sizeof c) & 0; }\n")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", root, str(src)],
                   check=True)


def test_planner_properties_over_random_shapes(lib):
    """The plan is a pure function of the shape: slice counts stay in range and keep at least 512 of K each,
    the workspace request matches the slices, huge grids are refused; 300 seeded shapes, no device needed."""
    import numpy as np
    rng = np.random.default_rng(2024)
    for _ in range(300):
        M, N = int(rng.integers(1, 9000)), int(rng.integers(1, 9000))
        K = int(2 ** rng.uniform(0, 17))
        batch = int(rng.choice([1, 1, 1, 2, 7, 64]))
        s = binding.auto_split_k(M, N, K, batch)
        assert 1 <= s <= 64, (M, N, K, batch, s)
        assert s == 1 or K // s >= 256, (M, N, K, batch, s)              # slices of 512 wanted, rounding may shave
        assert s == binding.auto_split_k(M, N, K, batch)                 # no hidden state
        need = binding.workspace_bytes(M, N, K, batch, "auto", 0)
        assert need in (0, s * batch * M * N * 4) or need >= batch * M * N * 4 * 2, (M, N, K, batch, s, need)
        assert binding.workspace_bytes(M, N, K, batch, "direct", 0) == 0
    # many output tiles are never sliced, one tile with a long K always is
    assert binding.auto_split_k(8192, 8192, 65536) == 1
    assert binding.auto_split_k(128, 128, 65536) > 8
