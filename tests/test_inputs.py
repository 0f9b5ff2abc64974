"""The seeded input generator: reproducible, sliceable, right distributions."""
import numpy as np

from paper_2604_01489_amd import inputs as gen


def test_counter_based_slices_agree():
    full = gen.normal(7, gen.STREAM_A, 5000, 0.5)
    part = gen.normal(7, gen.STREAM_A, 100, 0.5, start=1234)
    assert np.array_equal(full[1234:1334], part)
    u = gen.uniform(7, gen.STREAM_B, 5000, -1, 1)
    assert np.array_equal(u[4000:4010], gen.uniform(7, gen.STREAM_B, 10, -1, 1, start=4000))
    assert not np.array_equal(u[:100], gen.uniform(8, gen.STREAM_B, 100, -1, 1))
    assert not np.array_equal(u[:100], gen.uniform(7, gen.STREAM_A, 100, -1, 1))


def test_splitmix64_reference_words():
    """mix64 applied to the running counter must reproduce splitmix64's published
    first outputs for seed 0 (Steele, Lea, Flood; also the xoshiro seeding code)."""
    z = (np.arange(1, 4, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15))
    got = gen._mix64(z)
    assert [int(x) for x in got] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_distributions():
    x = gen.normal(1, 0, 1 << 18, 1.0).astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1) < 0.01
    assert abs(np.mean(x ** 3)) < 0.03 and abs(np.mean(x ** 4) - 3) < 0.1
    u = gen.uniform(1, 0, 1 << 18, -0.1, 0.1).astype(np.float64)
    assert u.min() >= -0.1 and u.max() <= 0.1 and abs(u.mean()) < 1e-3
    assert abs(u.var() - 0.2 ** 2 / 12) < 1e-4


def test_bf16_rounding_is_nearest_even():
    import torch
    x = gen.normal(3, 0, 100000, 3.0)
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(gen.to_bf16_bits(x), want)
    ties = np.array([1.00390625, 1.01171875, -1.00390625], dtype=np.float32)  # halfway cases
    assert [hex(v) for v in gen.to_bf16_bits(ties)] == ["0x3f80", "0x3f82", "0xbf80"]
    assert np.array_equal(gen.bf16_bits_to_f32(gen.to_bf16_bits(x)),
                          torch.from_numpy(x).to(torch.bfloat16).float().numpy())


def test_workload_table_matches_configs():
    w = gen.WORKLOADS
    assert (w["c1_f32_256"].M, w["c1_f32_256"].dtype, w["c1_f32_256"].seed) == (256, "f32", 0)
    c3 = w["c3_bf16_8192_bias_gelu"]
    assert (c3.M, c3.N, c3.K, c3.alpha, c3.act, c3.bias) == (8192, 8192, 8192, 0.5, "gelu_tanh", (-0.1, 0.1))
    assert c3.flops == 2 * 8192 ** 3
    c4 = w["c4_bf16_batched_512x512x64"]
    assert (c4.batch, c4.M, c4.N, c4.K) == (256, 512, 512, 64)
    assert abs(c4.algorithmic_bytes - 302e6) < 1e6
    c5 = w["c5_bf16_splitk_1024x1024x65536"]
    assert c5.alpha == 1 / 256 and c5.K == 65536


def test_operand_rows_can_be_regenerated():
    w = gen.WORKLOADS["c4_bf16_batched_512x512x64"]
    a = gen.make_operand(w, "A", batch_index=3)
    assert a.shape == (512, 64) and a.dtype == np.uint16
    assert np.array_equal(a[100:104], gen.make_operand(w, "A", 100, 4, batch_index=3))
    assert not np.array_equal(a, gen.make_operand(w, "A", batch_index=4))
