"""Search over the plan of one bf16 GEMM shape: structure first, by timing; counters later, to
break ties.

The paper's refinement loop withholds profiler feedback until the structure of a kernel has
settled ("Delayed Integration of Profiling Feedback"): structure first, counters later.  The
non-LLM analogue kept here is a small search over the structural choices this library leaves open
per shape -- the block tile and how many K slices -- timed with HIP events on the device.  Only
when the two fastest structures are within a few per cent of each other, which a timing on a shared
machine cannot separate, are hardware counters read: each of the two is run once more under
``rocprofv3 --pmc`` (a child process) and the one that moves fewer bytes beyond the L2s wins, the
traffic of every kernel of the call counted (a split plan pays for its partial tiles there).

    python -m paper_2604_01489_amd.tune M N K [batch] [--tie F]  the table, the tie-break, the library's own choice
    python -m paper_2604_01489_amd.tune --calibrate [--json FILE] [--write]
                                                               the rates of the planner's cost model, measured
                                                               (--write: into csrc/plan_rates.h; --json: the record)
    python -m paper_2604_01489_amd.tune --write-rates FILE     csrc/plan_rates.h from such a record

It is a tool for checking the fixed planning rules (and for callers who want to pass ``plan`` and
``split_k`` to ``gemm_epilogue_bf16_ex`` themselves), not part of the hot path.
"""
from __future__ import annotations

import csv
import glob
import os
import subprocess
import sys
import tempfile

from . import binding

TIE = 0.03          # structures closer than this in time are a tie for the clock
# what the same counters read for a plain device-to-device copy of known size: FETCH_SIZE reports
# half the bytes read, WRITE_SIZE the bytes written (KiB per dispatch)
FETCH_SCALE, WRITE_SCALE = 2.0, 1.0


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


def run_one(M: int, N: int, K: int, batch: int, tile: str, split: int, reps: int = 3):
    """One structure, a few launches and nothing else: what the counter run executes."""
    import torch
    dev = torch.device("cuda:0")
    A = torch.randn(batch * M, K, device=dev).to(torch.bfloat16).view(torch.int16)
    B = torch.randn(batch * K, N, device=dev).to(torch.bfloat16).view(torch.int16)
    C = torch.empty(batch * M, N, device=dev)
    binding.set_option("force_config", tile)
    for _ in range(reps):
        binding.gemm_epilogue_bf16_ex(M, N, K, A, K, B, N, None, 1.0, "none", C, N, batch,
                                      plan="direct" if split == 1 else "splitk", split_k=split)
    torch.cuda.synchronize()


def bytes_beyond_l2(counter_csv: str, reps: int) -> float:
    """HBM-side bytes per call from a rocprofv3 counter file: FETCH_SIZE and WRITE_SIZE (KiB per
    dispatch) of every library kernel, summed over the dispatches of a call."""
    total = 0.0
    with open(counter_csv, newline="") as fh:
        for row in csv.DictReader(fh):
            if "ge::" not in row["Kernel_Name"]:
                continue
            scale = {"FETCH_SIZE": FETCH_SCALE, "WRITE_SIZE": WRITE_SCALE}.get(row["Counter_Name"])
            if scale is not None:
                total += float(row["Counter_Value"]) * 1024.0 * scale
    return total / reps


def counters_for(M: int, N: int, K: int, batch: int, tile: str, split: int, workdir: str) -> float:
    """Run one structure under ``rocprofv3 --pmc`` in a child process (the interpreter itself after
    ``--``, as the profiler wants it) and return its bytes beyond the L2s.  One run per counter: the two
    together need more L2 counter slots than one pass has."""
    reps = 3
    total = 0.0
    for counter in ("FETCH_SIZE", "WRITE_SIZE"):
        out = os.path.join(workdir, f"pmc_{tile}_{split}_{counter}")
        cmd = ["rocprofv3", "--pmc", counter, "-d", out, "-o", "c", "--output-format", "csv", "--",
               sys.executable, "-m", "paper_2604_01489_amd.tune", "--one", str(M), str(N), str(K), str(batch), tile, str(split)]
        res = subprocess.run(cmd, capture_output=True, text=True, timeout=120,
                             cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
        files = glob.glob(os.path.join(out, "**", "*counter_collection.csv"), recursive=True)
        if res.returncode != 0 or not files:
            raise RuntimeError(f"counter run failed ({res.returncode}): {res.stderr[-400:]}")
        total += bytes_beyond_l2(files[0], reps)
    return total


def choose_structure(M: int, N: int, K: int, batch: int = 1, workdir: str | None = None):
    """Structure first: the timed search.  Counters later: if the runner-up is within TIE of the fastest,
    both are run under the profiler and the one with less traffic beyond the L2s is chosen.
    Returns (chosen (tile, split, us), reason, own, table, counters or None)."""
    best, own, table = sweep_structure(M, N, K, batch)
    ranked = sorted(table, key=lambda t: t[2])
    if len(ranked) < 2 or ranked[1][2] > (1.0 + TIE) * ranked[0][2]:
        return best, "fastest by more than the tie margin: no counters read", own, table, None
    with tempfile.TemporaryDirectory(dir=workdir) as tmp:
        traffic = [(c, counters_for(M, N, K, batch, c[0], c[1], tmp)) for c in ranked[:2]]
    chosen = min(traffic, key=lambda t: t[1])[0]
    return chosen, "tie in time, broken by bytes beyond the L2s", own, table, traffic


# ---- the planner's cost model, measured -----------------------------------------------------------
def _time_us(M, N, K, tile, plan, split, reps=20, warmup=5, batch=1):
    import torch
    dev = torch.device("cuda:0")
    A = torch.randn(batch * M, K, device=dev).to(torch.bfloat16).view(torch.int16)
    B = torch.randn(batch * K, N, device=dev).to(torch.bfloat16).view(torch.int16)
    C = torch.empty(batch * M, N, device=dev)
    binding.set_option("force_config", tile)
    try:
        def call():
            binding.gemm_epilogue_bf16_ex(M, N, K, A, K, B, N, None, 1.0, "none", C, N, batch, plan=plan, split_k=split)
        best = None
        for _ in range(3):                      # the least disturbed of three measurements
            for _ in range(warmup):
                call()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                call()
            e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1) / reps * 1e3
            best = t if best is None else min(best, t)
        return best
    finally:
        binding.set_option("force_config", None)


def calibrate():
    """The rates of ``plan_cost_us`` (csrc/gemm_epilogue_api.hip), each from two timings that differ in
    one quantity.  Per 32-wide K step and per launch (what a launch of one round costs beyond its steps):
    two K extents of a launch with 256 x 256 blocks one to a CU, of one with 128 x 128 blocks alone on
    their CUs and of one with two sharing a CU.  Per further round of blocks: a short-K batch of several
    rounds against the same batch four times as large.  The second pass of K slices: its launch from a
    sliced call against the direct call over one slice's K extent, its bytes per microsecond from the
    duration of the second kernel under the profiler's kernel trace (a child process)."""
    out = {}

    def line(tile, M, N, k1, k2):
        t1, t2 = _time_us(M, N, k1, tile, "direct", 1), _time_us(M, N, k2, tile, "direct", 1)
        step = (t2 - t1) / ((k2 - k1) / 32.0)
        return step, t1 - step * (k1 / 32.0), (t1, t2)

    def per_round(tile, blocks_per_round, step):
        # 512 x 512 x 64 per batch (four 256 blocks or sixteen 128 blocks), 128 and 512 batches: both
        # write more than the 256 MB memory-side cache holds, as a launch of many rounds does
        per_batch = 4 if tile == "256x256" else 16
        t_lo = _time_us(512, 512, 64, tile, "direct", 1, batch=128)
        t_hi = _time_us(512, 512, 64, tile, "direct", 1, batch=512)
        rounds = (512 - 128) * per_batch / blocks_per_round
        return (t_hi - t_lo) / rounds - 2.0 * step, (t_lo, t_hi)

    out["step256"], out["fixed256"], raw256 = line("256x256", 4096, 4096, 2048, 8192)         # 256 blocks: one to a CU
    out["step128_alone"], out["fixed128_alone"], raw128a = line("128x128", 2048, 2048, 2048, 8192)   # 256 blocks of 128
    out["step128_shared"], out["fixed128_shared"], raw128s = line("128x128", 4096, 2048, 2048, 8192)  # 512 blocks: two to a CU
    out["round256"], rawr256 = per_round("256x256", 256, out["step256"])
    out["round128_shared"], rawr128 = per_round("128x128", 512, out["step128_shared"])
    # the second launch: one tile, two slices of 4096 against the direct call over 4096
    pair_small = _time_us(128, 128, 8192, "128x128", "splitk", 2)
    direct_small = _time_us(128, 128, 4096, "128x128", "direct", 1)
    out["second_pass_launch"] = max(pair_small - direct_small, 0.5)
    M = N = 1024
    K, S, reps = 65536, 16, 10
    with tempfile.TemporaryDirectory() as tmp:
        cmd = ["rocprofv3", "--kernel-trace", "--stats", "-d", tmp, "-o", "c", "--output-format", "csv", "--",
               sys.executable, "-m", "paper_2604_01489_amd.tune", "--one", str(M), str(N), str(K), "1", "256x256", str(S), str(reps)]
        res = subprocess.run(cmd, capture_output=True, text=True, timeout=180,
                             cwd=os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
        files = glob.glob(os.path.join(tmp, "**", "*kernel_stats.csv"), recursive=True)
        if res.returncode != 0 or not files:
            raise RuntimeError(f"kernel trace failed ({res.returncode}): {res.stderr[-400:]}")
        reduce_us = None
        with open(files[0], newline="") as fh:
            for row in csv.DictReader(fh):
                if "splitk_reduce_kernel" in row["Name"]:
                    # the mean without the slowest dispatch (the first one runs before the clocks have settled)
                    reduce_us = (float(row["TotalDurationNs"]) - float(row["MaxNs"])) / max(int(row["Calls"]) - 1, 1) / 1e3
    if reduce_us is None:
        raise RuntimeError("the kernel trace does not name the second kernel of the split plan")
    out["second_pass_bytes_per_us"] = (S + 1) * M * N * 4.0 / reduce_us
    out["raw"] = {"256": raw256, "128_alone": raw128a, "128_shared": raw128s, "rounds256": rawr256, "rounds128_shared": rawr128,
                  "second_launch": {"pair_us": pair_small, "direct_us": direct_small}, "reduce_us": reduce_us}
    return out


RATES_HEADER = """// Rates of the planner's cost model (plan_cost_us in gemm_epilogue_api.hip), in microseconds.
// GENERATED by `python -m paper_2604_01489_amd.tune --calibrate --write` on one MI355X; the run that
// produced these numbers is kept with the profile summaries.  The model ranks structures,
// it does not predict times: regenerate on a part whose clocks differ, do not edit by hand.
#pragma once

namespace ge_host {{

constexpr double kStep256Us = {step256:.3f};          // 256 x 256 block, one to a CU: per 32-wide K step
constexpr double kFixed256Us = {fixed256:.2f};        //   ... and per launch of one round (launch, pipeline fill, tile store)
constexpr double kRound256Us = {round256:.2f};        //   ... and per further round of blocks
constexpr double kStep128AloneUs = {step128_alone:.3f};     // 128 x 128 block alone on a CU
constexpr double kFixed128AloneUs = {fixed128_alone:.2f};
constexpr double kStep128SharedUs = {step128_shared:.3f};    // two 128 x 128 blocks sharing a CU, per round of two
constexpr double kFixed128SharedUs = {fixed128_shared:.2f};
constexpr double kRound128SharedUs = {round128_shared:.2f};
constexpr double kSecondPassLaunchUs = {second_pass_launch:.2f};      // K slices: the second launch
constexpr double kSecondPassBytesPerUs = {second_pass_bytes_per_us:.4g};  //   ... and its partial tiles, written and read

}}  // namespace ge_host
"""


def write_rates(rates, path=None):
    path = path or os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "plan_rates.h")
    with open(path, "w") as fh:
        fh.write(RATES_HEADER.format(**rates))
    return path


if __name__ == "__main__":
    argv = sys.argv[1:]
    if argv and argv[0] == "--one":
        M, N, K, batch = (int(x) for x in argv[1:5])
        run_one(M, N, K, batch, argv[5], int(argv[6]), *(int(x) for x in argv[7:8]))
        sys.exit(0)
    if argv and argv[0] == "--calibrate":
        import json
        rates = calibrate()
        for k, v in rates.items():
            print(f"{k}: {v}")
        if "--json" in argv:                 # the record of the run, to be kept with the profiles
            with open(argv[argv.index("--json") + 1], "w") as fh:
                json.dump(rates, fh, indent=1)
        if "--write" in argv:
            print("written:", write_rates(rates))
        sys.exit(0)
    if argv and argv[0] == "--write-rates":  # the header from the record of a calibration run
        import json
        with open(argv[1]) as fh:
            print("written:", write_rates(json.load(fh)))
        sys.exit(0)
    if "--tie" in argv:                # a wider tie margin, to see the counters at work on any shape
        i = argv.index("--tie")
        TIE = float(argv[i + 1])
        del argv[i:i + 2]
    dims = [int(x) for x in argv]
    if len(dims) not in (3, 4):
        sys.exit("usage: python -m paper_2604_01489_amd.tune M N K [batch] | --calibrate [--write]")
    chosen, reason, own, table, traffic = choose_structure(*dims)
    best = min(table, key=lambda t: t[2])
    for tile, s, us in table:
        print(f"tile {tile}  split_k {s:3d}: {us:9.1f} us" + ("   <- fastest" if (tile, s, us) == best else ""))
    if traffic:
        for (tile, s_, us), nbytes in traffic:
            print(f"counters: tile {tile} split_k {s_}: {nbytes / 1e6:.1f} MB beyond the L2s per call")
    print(f"chosen: tile {chosen[0]} split_k {chosen[1]} ({reason})")
    print(f"the library's own plan: {own[0]}  {own[1]:.1f} us")
