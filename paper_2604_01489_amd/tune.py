"""Search over the plan of one bf16 GEMM shape by timing alone.

The paper's refinement loop withholds profiler feedback until the structure of a kernel has
settled ("Delayed Integration of Profiling Feedback"): structure first, counters later.  The
non-LLM analogue kept here is a small search over the structural choices this library leaves open
per shape -- the block tile and how many K slices -- timed with HIP events on the device; no
counters are read.
``python -m paper_2604_01489_amd.tune M N K [batch]`` prints the table and the library's own choice.
It is a tool for checking the fixed planning rules (and for callers who want to pass ``plan`` and
``split_k`` to ``gemm_epilogue_bf16_ex`` themselves), not part of the hot path.
"""
from __future__ import annotations

import sys

from . import binding


def candidate_splits(K: int, limit: int = 64):
    """1 (direct) and the slice counts that keep at least 256 of K per slice, roughly x1.5 apart."""
    out, s = [1], 2
    while s <= limit and K // s >= 256:
        out.append(s)
        s = max(s + 1, int(s * 1.5))
    return out


def sweep_split_k(M: int, N: int, K: int, batch: int = 1, warmup: int = 5, reps: int = 30):
    """Time every candidate; returns (best_split, auto_split, [(split, microseconds), ...])."""
    import torch
    dev = torch.device("cuda:0")
    A = torch.randn(batch * M, K, device=dev).to(torch.bfloat16).view(torch.int16)
    B = torch.randn(batch * K, N, device=dev).to(torch.bfloat16).view(torch.int16)
    C = torch.empty(batch * M, N, device=dev)
    table = []
    auto = binding.auto_split_k(M, N, K, batch)
    for s in sorted(set(candidate_splits(K)) | {auto}):
        plan = "direct" if s == 1 else "splitk"

        def call():
            binding.gemm_epilogue_bf16_ex(M, N, K, A, K, B, N, None, 1.0, "none", C, N, batch, plan=plan, split_k=s)

        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        table.append((s, e0.elapsed_time(e1) / reps * 1e3))
    best = min(table, key=lambda t: t[1])[0]
    return best, auto, table


def sweep_structure(M: int, N: int, K: int, batch: int = 1, warmup: int = 5, reps: int = 20):
    """The two structural choices together: block tile (256 x 256 or 128 x 128, forced through the
    library's "force_config" option for the duration of a timing) and the number of K slices.
    Returns (fastest (tile, split, us), the library's own (kernel name, us), [(tile, split, us), ...])."""
    import torch
    dev = torch.device("cuda:0")
    A = torch.randn(batch * M, K, device=dev).to(torch.bfloat16).view(torch.int16)
    B = torch.randn(batch * K, N, device=dev).to(torch.bfloat16).view(torch.int16)
    C = torch.empty(batch * M, N, device=dev)

    def timed(plan, s):
        def call():
            binding.gemm_epilogue_bf16_ex(M, N, K, A, K, B, N, None, 1.0, "none", C, N, batch, plan=plan, split_k=s)
        for _ in range(warmup):
            call()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            call()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    binding.set_option("force_config", None)
    try:
        own_us = timed("auto", 0)
        own = (binding.last_config(), own_us)
        table = []
        for tile in ("256x256", "128x128"):
            binding.set_option("force_config", tile)
            for s in candidate_splits(K):
                table.append((tile, s, timed("direct" if s == 1 else "splitk", s)))
    finally:
        binding.set_option("force_config", None)
    return min(table, key=lambda t: t[2]), own, table


if __name__ == "__main__":
    dims = [int(x) for x in sys.argv[1:]]
    if len(dims) not in (3, 4):
        sys.exit("usage: python -m paper_2604_01489_amd.tune M N K [batch]")
    best, own, table = sweep_structure(*dims)
    for tile, s, us in table:
        print(f"tile {tile}  split_k {s:3d}: {us:9.1f} us" + ("   <- fastest" if (tile, s, us) == best else ""))
    print(f"the library's own plan: {own[0]}  {own[1]:.1f} us")
