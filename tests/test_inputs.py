"""The seeded generators: deterministic, right shapes, right distributions."""
import numpy as np

import mqa_inputs as mi


def test_streams_are_reproducible_and_distinct():
    a = mi.rng(4, 7).standard_normal(8)
    assert np.array_equal(a, mi.rng(4, 7).standard_normal(8))
    assert not np.array_equal(a, mi.rng(4, 8).standard_normal(8))
    assert not np.array_equal(a, mi.rng(5, 7).standard_normal(8))


def test_bf16_plumbing_round_trip():
    x = np.array([1.0, -2.5, 3.140625, 0.0], dtype=np.float32)
    bits = mi.f32_to_bf16_bits(x)
    assert bits.dtype == np.uint16
    assert np.array_equal(mi.bf16_bits_to_f32(bits), x)          # all exactly representable
    assert np.array_equal(mi.bits_to_torch_bf16(bits).float().numpy(), x)
    assert mi.f32_to_bf16_bits(np.array([1.00390625], np.float32))[0] == 0x3F80   # tie -> even


def test_config1_and_2_shapes_and_scale():
    c = mi.config1()
    assert c["x"].shape == (1, 1024) and c["M"].shape == (1, 128, 1024)
    assert c["P_q"].shape == (8, 1024, 128) and c["P_k"].shape == (1024, 128) and c["P_o"].shape == (8, 1024, 128)
    assert abs(c["P_q"].std() * 32 - 1) < 0.01 and c["x"].dtype == np.float32
    c = mi.config2(b=4, steps=3)
    assert c["X"].shape == (4, 3, 1024) and abs(c["X"].std() - 1) < 0.05
    assert abs(c["P_k"].std() * 32 - 1) < 0.02


def test_config4_blocks():
    K, V = mi.config4_kv(b=2, m=64, threads=2)
    assert K.shape == (2, 64, 128) and K.dtype == np.uint16
    K2, _ = mi.config4_kv(b=1, m=64, threads=1)
    assert np.array_equal(K[0], K2[0])                    # per-sequence streams
    assert abs(mi.bf16_bits_to_f32(K).std() - 1) < 0.05
    q = mi.config4_q(b=2)
    assert q.shape == (2, 32, 128) and abs(q.std() * np.sqrt(128) - 1) < 0.05
    Kh, Vh = mi.config4_kv_mh_block(1, 3, m=16)
    assert Kh.shape == (16, 128) and not np.array_equal(Kh, mi.config4_kv_mh_block(1, 4, m=16)[0])


def test_config5_ragged_and_outliers():
    q, K, V, lens = mi.config5(b=6, h=4, cap=512, outlier_fraction=0.05)
    assert lens.dtype == np.int32 and lens.min() >= 1 and lens.max() <= 512
    Kf = mi.bf16_bits_to_f64(K)
    boosted = 0
    for i in range(6):
        L = int(lens[i])
        assert not np.isnan(Kf[i, :L]).any() and np.isnan(Kf[i, L:]).all()
        logits = Kf[i, :L] @ q[i].astype(np.float64).T          # [L, h] plain dot products
        boosted += int((logits.max(axis=1) > 25).sum())
    assert boosted >= 1                                          # forced-large logits are present
    assert np.isnan(mi.bf16_bits_to_f64(V)[0, int(lens[0]):]).all() or lens[0] == 512


def test_random_case_modes():
    c = mi.random_case(1, b=5, h=2, cap=9, k=8, v=8, lens="with_zero")
    assert (c["lens"] == 0).any() and c["K"].dtype == np.uint16
    c = mi.random_case(2, b=2, h=3, cap=4, k=8, v=16, cache="f32", multi_head=True, lens=[4, 2])
    assert c["K"].shape == (2, 3, 4, 8) and c["V"].shape == (2, 3, 4, 16)
    assert np.isnan(c["K"][1, :, 2:]).all() and not np.isnan(c["K"][1, :, :2]).any()
