"""Host logic: the seeded input generator and the workload table."""
import numpy as np

from paper_2409_18747_amd import workloads


def test_draw_is_deterministic_and_ordered():
    a = workloads.draw(2, 3, 5, 8, "bf16", seed=7)
    b = workloads.draw(2, 3, 5, 8, "bf16", seed=7)
    for k in ("Q", "K", "V", "dO", "s"):
        np.testing.assert_array_equal(a[k], b[k])
    c = workloads.draw(2, 3, 5, 8, "bf16", seed=8)
    assert not np.array_equal(a["Q"], c["Q"])
    # dropping dO does not shift the draw of s
    d = workloads.draw(2, 3, 5, 8, "bf16", seed=7, with_dO=False)
    np.testing.assert_array_equal(a["s"], d["s"])
    assert "dO" not in d
    assert a["s"].min() >= 0.5 and a["s"].max() <= 1.5


def test_bf16_rounding_is_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -7, -0.3, 3.0e38],
                 dtype=np.float32)
    r = workloads.round_to_bf16(x)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0); 1 + 3*2^-8 ties up
    np.testing.assert_array_equal(r[:4], np.array([1.0, 1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7],
                                                  dtype=np.float32))
    bits = workloads.f32_to_bf16_bits(r)
    np.testing.assert_array_equal(workloads.bf16_bits_to_f32(bits), r)
    assert np.all((r.view(np.uint32) & 0xFFFF) == 0)
    assert abs(r[4] + 0.3) <= 0.3 * 2.0 ** -8


def test_value_scale_and_statistics():
    x = workloads.draw(1, 2, 4096, 64, "f32", seed=3, value_scale=0.5)
    assert abs(float(x["Q"].std()) - 0.5) < 0.01
    assert abs(float(x["V"].mean())) < 0.01


def test_workload_table_matches_the_benchmark_shapes():
    w = workloads.WORKLOADS
    assert (w["cfg1_small_causal_fwd_f32"].B, w["cfg1_small_causal_fwd_f32"].N,
            w["cfg1_small_causal_fwd_f32"].d, w["cfg1_small_causal_fwd_f32"].dtype) == (1, 256, 32, "f32")
    g = w["cfg2_gpt_causal_fwdbwd_bf16"]
    assert (g.B, g.H, g.N, g.d, g.dtype, g.seed, g.causal) == (8, 12, 1024, 64, "bf16", 1, True)
    b = w["cfg3_bert_bidir_fwdbwd_bf16"]
    assert (b.B, b.H, b.N, b.d, b.causal) == (32, 12, 512, 64, False)
    l = w["cfg4_long_causal_fwdbwd_bf16"]
    assert (l.B, l.H, l.N, l.value_scale) == (1, 16, 65536, 0.5)
    dcd = w["cfg5_decode_bf16"]
    assert (dcd.B, dcd.H, dcd.N, dcd.d, dcd.extra["steps"]) == (256, 16, 2048, 128, 4096)
    q, k, v = workloads.draw_tokens(2, 3, 4, 8, "bf16", seed=4)
    assert q.shape == (4, 2, 3, 8) and not np.array_equal(q, k)
