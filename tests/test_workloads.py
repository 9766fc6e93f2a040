"""The seeded input generator: determinism and the stated distributions."""
import numpy as np

import workloads as W


def test_deterministic_and_tensor_ids_differ():
    a = W.fill(1, 2, 64, 32, seed=7, tensor_id=W.TENSOR_Q)
    b = W.fill(1, 2, 64, 32, seed=7, tensor_id=W.TENSOR_Q)
    c = W.fill(1, 2, 64, 32, seed=7, tensor_id=W.TENSOR_K)
    assert np.array_equal(a, b) and not np.array_equal(a, c)


def test_normal_moments_and_t3_tails():
    x = W.bf16_bits_to_f32(W.fill(1, 4, 4096, 64, seed=1, tensor_id=1)).astype(np.float64)
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    t = W.bf16_bits_to_f32(W.fill(1, 4, 4096, 64, seed=1, tensor_id=1, dist="t3", scale=0.5))
    t = t.astype(np.float64)
    # Student-t(3) scaled by 0.5: median |x| = 0.5 * 0.7649, P(|t3| > 5.841) = 0.01
    assert abs(np.median(np.abs(t)) - 0.5 * 0.7649) < 0.01
    assert abs((np.abs(t) > 0.5 * 5.841).mean() - 0.01) < 0.002


def test_outlier_channels_and_tokens():
    w = W.CONFIGS[2]
    k = W.bf16_bits_to_f32(W.fill(1, 2, 2048, 128, seed=2, tensor_id=W.TENSOR_K,
                                  n_chan=4, chan_mult=20.0)).astype(np.float64)
    sd = k.std(axis=2)                                   # [1, 2, 128]
    assert ((sd > 10).sum(-1) == 4).all() and ((sd < 1.2) | (sd > 10)).all()
    q = W.bf16_bits_to_f32(W.fill(1, 1, 20000, 16, seed=3, tensor_id=1, tok_mod=100, tok_mult=10.0))
    v = W.bf16_bits_to_f32(W.fill(1, 1, 20000, 16, seed=3, tensor_id=3, tok_mod=100, tok_mult=10.0))
    rq = np.abs(q[0, 0]).mean(-1) > 4; rv = np.abs(v[0, 0]).mean(-1) > 4
    assert 0.005 < rq.mean() < 0.015 and np.array_equal(rq, rv)     # same token set, ~1 %
    assert w.k_outlier_channels == 4


def test_bf16_round_trip_helpers():
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    b = W.f32_to_bf16_bits(x)
    import torch
    assert np.array_equal(W.bf16_bits_to_f32(b),
                          torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy())


def test_config_table_matches_benchmark_shapes():
    shapes = [(w.B, w.Hq, w.Hkv, w.L, w.d, w.causal) for w in W.CONFIGS]
    assert shapes == [(1, 2, 2, 256, 64, False), (2, 12, 12, 32760, 128, False),
                      (4, 32, 8, 4096, 128, True), (1, 40, 40, 75600, 128, False),
                      (1, 64, 8, 32768, 128, True)]
    assert abs(W.CONFIGS[3].fwd_flops - 117.05e12) / 117.05e12 < 1e-3
