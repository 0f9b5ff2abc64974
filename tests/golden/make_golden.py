"""Writes the stored expected values of tests/golden/*.txt.  Calls only oracle/ and the seeded input
generator: no value here ever comes from the GPU library.  The paper prints no worked numeric
example of the operator, so these files are not the paper's numbers; they freeze what the pinned
oracles return on three small seeded cases, so that a later change to an oracle's arithmetic
cannot pass unnoticed (tests/test_golden.py).  Run from the repository root:

    python tests/golden/make_golden.py
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle                                              # noqa: E402
from paper_2604_01489_amd import inputs as gen            # noqa: E402

HERE = os.path.dirname(os.path.abspath(__file__))


def cases():
    """name -> fp64 array, each from one oracle on seeded bf16 inputs."""
    M, N, K = 5, 7, 12
    A = gen.to_bf16_bits(gen.normal(100, gen.STREAM_A, M * K, 1.0).reshape(M, K))
    B = gen.to_bf16_bits(gen.normal(100, gen.STREAM_B, K * N, 1.0).reshape(K, N))
    bias = gen.uniform(100, gen.STREAM_BIAS, N, -1.0, 1.0)
    out = {"gemm_epilogue_5x7x12_gelu": oracle.gemm_epilogue(A, B, bias, 0.5, "gelu_tanh")}
    rs = gen.uniform(100, gen.STREAM_ROW_SCALE, M, 0.5, 1.5)
    R = gen.to_bf16_bits(gen.uniform(100, gen.STREAM_RESIDUAL, M * N, -1.0, 1.0).reshape(M, N))
    out["gemm_fused_5x7x12_tn_chain_bf16"] = oracle.gemm_fused(
        M, N, K, np.ascontiguousarray(A.T), B, transA=True, alpha=0.75, row_scale=rs, bias=bias, residual=R,
        beta=-0.5, act="relu", clamp=(0.1, 2.0), out="bf16")[0]
    X = gen.to_bf16_bits(gen.normal(101, gen.STREAM_A, 1 * 5 * 6 * 4, 1.0).reshape(1, 5, 6, 4))
    Wt = gen.to_bf16_bits(gen.normal(101, gen.STREAM_B, 3 * 2 * 3 * 4, 0.2).reshape(3, 2, 3, 4))
    cb = gen.uniform(101, gen.STREAM_BIAS, 3, -1.0, 1.0)
    out["conv2d_1x5x6x4_to_3_k2x3_s2x1_p1x2"] = oracle.conv2d_nhwc(
        X, Wt, stride=(2, 1), pad=(1, 2), alpha=1.5, bias=cb, act="gelu_tanh").reshape(-1, 3)
    return out


def write():
    for name, arr in cases().items():
        with open(os.path.join(HERE, name + ".txt"), "w") as f:
            f.write(f"# {name}: shape {arr.shape}, one row per line, C99 hex floats (exact fp64)\n")
            f.write("# written by tests/golden/make_golden.py from oracle/ alone; not the paper's numbers\n")
            for row in np.atleast_2d(arr):
                f.write(" ".join(float(v).hex() for v in row) + "\n")


if __name__ == "__main__":
    write()
