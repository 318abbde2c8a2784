"""The synthetic input generator: determinism, slice independence, statistics."""
import math

import numpy as np

import synth


def test_streams_are_deterministic_and_distinct():
    a = synth.latent_weights(0, 64, 128, layer=2, matrix="o")
    b = synth.latent_weights(0, 64, 128, layer=2, matrix="o")
    c = synth.latent_weights(0, 64, 128, layer=3, matrix="o")
    d = synth.latent_weights(1, 64, 128, layer=2, matrix="o")
    assert np.array_equal(a, b)
    assert not np.array_equal(a, c) and not np.array_equal(a, d)


def test_rows_can_be_generated_independently():
    full = synth.activations_bf16(5, 8, 256)
    part = synth.activations_bf16(5, 3, 256, row0=4)
    assert np.array_equal(full[4:7], part)


def test_weight_statistics():
    W = synth.latent_weights(0, 1024, 1024)
    assert W.dtype == np.float32
    n = W.size
    assert abs(W.mean()) < 5 * 0.02 / math.sqrt(n)
    assert abs(W.std() - 0.02) < 5 * 0.02 / math.sqrt(2 * n)
    # kurtosis of a normal: 3
    z = W.astype(np.float64) / 0.02
    assert abs((z ** 4).mean() - 3.0) < 0.05


def test_activation_recipe():
    K = 2560
    ch = synth.outlier_channels(0, K)
    assert ch.size == 26 and len(set(ch.tolist())) == 26 and ch.min() >= 0 and ch.max() < K
    x = synth.bf16_bits_to_f32(synth.activations_bf16(0, 64, K))
    normal = np.ones(K, bool)
    normal[ch] = False
    assert abs(x[:, normal].std() - 1.0) < 0.02
    assert abs(x[:, ch].std() - 20.0) < 2.0
    assert synth.outlier_channels(0, 6912, matrix="down").size == 69
    r = synth.bf16_bits_to_f32(synth.activations_bf16(0, 16, 6912, matrix="down", relu2=True))
    assert r.min() >= 0 and abs((r == 0).mean() - 0.5) < 0.02


def test_uniform_i8_range():
    q = synth.uniform_i8(1, (4, 4096), -127, 127)
    assert q.min() == -127 and q.max() == 127
    t = synth.uniform_i8(1, (4, 4096), -1, 1)
    assert set(np.unique(t).tolist()) == {-1, 0, 1}
