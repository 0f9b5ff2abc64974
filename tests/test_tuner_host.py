"""Host-side checks of the tuner (paper_2604_01489_amd/tune.py): the counter file of the profiler is read
as documented, a tie in time is broken by traffic and a clear winner is not, and the generated header of
the planner's rates holds what the calibration record says."""
import os

import pytest

from paper_2604_01489_amd import tune

HEADER = ('"Correlation_Id","Dispatch_Id","Agent_Id","Queue_Id","Process_Id","Thread_Id","Grid_Size","Kernel_Id",'
          '"Kernel_Name","Workgroup_Size","LDS_Block_Size","Scratch_Size","VGPR_Count","Accum_VGPR_Count","SGPR_Count",'
          '"Counter_Name","Counter_Value","Start_Timestamp","End_Timestamp"\n')


def row(i, kernel, counter, value):
    return f'{i},{i},"Agent 1",1,7,7,512,6,"{kernel}",256,0,0,8,0,32,"{counter}",{value},1,2\n'


def test_counter_file_is_summed_per_call(tmp_path):
    f = tmp_path / "c_counter_collection.csv"
    gemm, red = "void ge::gemm_bf16_kernel<128, 128>(ge::GemmParams)", "ge::splitk_reduce_kernel(float const*)"
    text = HEADER + row(1, "__amd_rocclr_copyBuffer", "FETCH_SIZE", 999.0)
    for i in range(3):              # three calls of two kernels each
        text += row(2 + 2 * i, gemm, "FETCH_SIZE", 1000.0) + row(3 + 2 * i, red, "FETCH_SIZE", 24.0)
    f.write_text(text)
    # KiB per dispatch, FETCH_SIZE counts half the bytes: (1000 + 24) KiB * 2 per call; the copy is not ours
    assert tune.bytes_beyond_l2(str(f), 3) == pytest.approx((1000.0 + 24.0) * 1024 * 2.0)
    f.write_text(HEADER + row(1, gemm, "WRITE_SIZE", 512.0))
    assert tune.bytes_beyond_l2(str(f), 1) == pytest.approx(512.0 * 1024)


def test_ties_go_to_the_counters_and_clear_winners_do_not(monkeypatch):
    table = [("256x256", 1, 100.0), ("128x128", 1, 101.0), ("128x128", 2, 140.0)]
    monkeypatch.setattr(tune, "sweep_structure", lambda *a, **k: (table[0], ("own", 100.0), table))
    asked = []

    def fake_counters(M, N, K, batch, tile, split, workdir):
        asked.append((tile, split))
        return {"256x256": 9.0e8, "128x128": 5.0e8}[tile]

    monkeypatch.setattr(tune, "counters_for", fake_counters)
    chosen, reason, own, _, traffic = tune.choose_structure(1024, 1024, 1024)
    assert chosen == ("128x128", 1, 101.0) and "tie" in reason and sorted(asked) == [("128x128", 1), ("256x256", 1)]
    # the runner-up 10 % behind: the clock decides, the profiler is not started
    table[1] = ("128x128", 1, 110.0)
    asked.clear()
    chosen, reason, _, _, traffic = tune.choose_structure(1024, 1024, 1024)
    assert chosen == table[0] and traffic is None and not asked


def test_rates_header_is_generated_from_the_record(tmp_path):
    rates = dict(step256=0.65, fixed256=16.5, round256=11.25, step128_alone=0.24, fixed128_alone=8.9, step128_shared=0.47,
                 fixed128_shared=8.2, round128_shared=6.75, second_pass_launch=3.5, second_pass_bytes_per_us=5.6e6, raw={})
    path = tune.write_rates(rates, str(tmp_path / "plan_rates.h"))
    text = open(path).read()
    for needle in ("kStep256Us = 0.650", "kFixed256Us = 16.50", "kRound256Us = 11.25", "kStep128SharedUs = 0.470",
                   "kRound128SharedUs = 6.75", "kSecondPassBytesPerUs = 5.6e+06",
                   "GENERATED"):
        assert needle in text
    # the committed header has the same shape (the same names, generated the same way)
    committed = open(os.path.join(os.path.dirname(tune.__file__), "csrc", "plan_rates.h")).read()
    import re
    names = lambda t: re.findall(r"constexpr double (k\w+)", t)
    assert names(committed) == names(text) and "GENERATED" in committed
